// pamm_compress / pamm_compress_idx and their _eps forms: Alg. 1, procedure Compress.  With a finite tolerance
// (Eq. 2) the score kernel also sums ||X_i||^2 from the chunks of X as they pass through its registers, and the
// final decision drops the rows whose best representative is outside the neighbourhood.
//
// Launches on the caller's stream:
//   k_gather    C_j = X[idx_j] (bit copy), ||C_j||^2 in fp64, a content hash per generator (k_gather_arg: the same
//               with up to 512 sampled row numbers in the kernel's argument block)
//   k_score     streams X once; D = C X^T on the matrix cores with C staged through LDS, then per token the
//               largest values of s(i,j) = <X_i,C_j>^2/||C_j||^2 (Lemma 1) and where they occur.  With up to 256
//               generators (one column block) it also takes the final decision: f, alpha (Eq. 1), the few rows
//               whose leading scores are too close for fp32 to separate being re-decided in fp64
//   k_finalize  only with more than 256 generators: merges the column blocks and takes that final decision
#include <hip/hip_runtime.h>

#include "pamm_device.h"
#include "pamm_plan.h"
#include "pamm_profile.h"

namespace pamm {

// ------------------------------------------------------------------------------------------------
// Per-token record of the leading scores.  s1 > s2 > s3 > s4 are the four largest DISTINCT score values known;
// j1 / j2 / j3 are the lowest generator numbers attaining s1 / s2 / s3 (j3 = -1: the third value is known but not
// who attains it; s4 is a value only); d1 is the dot product behind s1; jt is the lowest generator other than j1
// that attains s1 exactly (-1 if none).  Bit-identical generators (padding tokens sampled twice) produce
// bit-identical scores, so they meet in jt instead of hiding the real runners-up.
struct Best {
    float s1; int j1; float d1; int jt; float s2; int j2; float s3; int j3; float s4;

    __device__ __forceinline__ void init() {
        s1 = -1.f; j1 = 0; d1 = 0.f; jt = -1; s2 = -2.f; j2 = 0; s3 = -3.f; j3 = -1; s4 = -4.f;
    }

    // A value below s1; j = -1 if it is not known who attains it.  Such a value never ranks second: in the record it
    // comes from, two larger values stand above it.
    __device__ __forceinline__ void insert_lower(float s, int j) {
        if (s > s2) { s4 = s3; s3 = s2; j3 = j2; s2 = s; j2 = j; }
        else if (s == s2) { if (j >= 0) j2 = min(j2, j); }
        else if (s > s3) { s4 = s3; s3 = s; j3 = j; }
        else if (s == s3) { j3 = (j3 < 0 || j < 0) ? max(j3, j) : min(j3, j); }
        else if (s > s4) { s4 = s; }
    }

    // union with a record built over a disjoint set of generators
    __device__ __forceinline__ void merge(const Best& o) {
        if (o.s1 > s1) {
            s4 = s3; s3 = s2; j3 = j2; s2 = s1; j2 = j1;
            s1 = o.s1; j1 = o.j1; d1 = o.d1; jt = o.jt;
        } else if (o.s1 == s1) {
            int lo = min(j1, o.j1), t = max(j1, o.j1);
            if (o.j1 < j1) d1 = o.d1;
            if (jt >= 0) t = min(t, jt);
            if (o.jt >= 0) t = min(t, o.jt);
            j1 = lo; jt = t;
        } else {
            insert_lower(o.s1, o.j1);
        }
        insert_lower(o.s2, o.j2);
        insert_lower(o.s3, o.j3);
        if (o.s4 < s3 && o.s4 > s4) s4 = o.s4;      // three larger values of o are already in: at best fourth
    }

    // 32-byte record: generator numbers fit 16 bits (k <= 16384); 0xffff stands for "none"
    __device__ __forceinline__ void store(u32x4_t* dst) const {
        dst[0] = u32x4_t{__float_as_uint(s1), __float_as_uint(d1), __float_as_uint(s2), __float_as_uint(s3)};
        dst[1] = u32x4_t{__float_as_uint(s4), uint32_t(j1) | (uint32_t(jt) << 16), uint32_t(j2) | (uint32_t(j3) << 16), 0u};
    }
    static __device__ __forceinline__ void store_norm(u32x4_t* dst, float nx) {      // ||X_i||^2 rides in the spare slot
        reinterpret_cast<float*>(dst + 1)[3] = nx;
    }
    static __device__ __forceinline__ float load_norm(const u32x4_t* src) { return __uint_as_float(src[1].w); }
    __device__ __forceinline__ void load(const u32x4_t* src) {
        const u32x4_t p = src[0], q = src[1];
        s1 = __uint_as_float(p.x); d1 = __uint_as_float(p.y); s2 = __uint_as_float(p.z); s3 = __uint_as_float(p.w);
        s4 = __uint_as_float(q.x);
        j1 = int(q.y & 0xffffu); jt = int(q.y >> 16); jt = jt == 0xffff ? -1 : jt;
        j2 = int(q.z & 0xffffu); j3 = int(q.z >> 16); j3 = j3 == 0xffff ? -1 : j3;
    }
};

// ------------------------------------------------------------------------------------------------
// k_gather: one workgroup per generator.  The row numbers come from memory (caller-chosen generators) or ride in the
// kernel's own argument block, kArgGenerators per launch (k_gather_arg): sampled indices then need no buffer that
// outlives the call, and a captured launch replays with the indices it was captured with.
constexpr int kArgGenerators = 512;
struct IdxByValue { int32_t v[kArgGenerators]; };

template <typename TR>
__device__ __forceinline__ void gather_row(const u32x4_t* __restrict__ X, int j, int src, int b, int nch, u32x4_t* __restrict__ C,
                                           int32_t* __restrict__ idx_out, float* __restrict__ inv, double* __restrict__ cn2,
                                           unsigned long long* __restrict__ hash, int32_t* __restrict__ eta) {
    if (eta && j == 0 && threadIdx.x == 0) *eta = 0;          // rows dropped by the neighbourhood condition: counted later
    src = src < 0 ? 0 : (src >= b ? b - 1 : src);
    const u32x4_t* xr = X + size_t(src) * nch;
    u32x4_t* cr = C + size_t(j) * nch;
    double acc = 0.0;
    unsigned long long h = 0;
    for (int c = threadIdx.x; c < nch; c += 256) {
        u32x4_t v = xr[c];
        cr[c] = v;
        float e[TR::kPerChunk];
        TR::unpack(v, e);
#pragma unroll
        for (int q = 0; q < TR::kPerChunk; ++q) acc += double(e[q]) * double(e[q]);
        // position-keyed 64-bit mix of the raw bits; summed, so the order of chunks does not matter
        unsigned long long z = (((unsigned long long)v.x << 32) | v.y) * 0x9E3779B97F4A7C15ULL
                             + (((unsigned long long)v.z << 32) | v.w) * 0xC2B2AE3D27D4EB4FULL
                             + (unsigned long long)(c + 1) * 0x165667B19E3779F9ULL;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
        h += z ^ (z >> 31);
    }
    acc = wave_sum(acc);
    h = wave_sum(h);
    __shared__ double sacc[4];
    __shared__ unsigned long long sh[4];
    if ((threadIdx.x & 63) == 0) { sacc[threadIdx.x >> 6] = acc; sh[threadIdx.x >> 6] = h; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = (sacc[0] + sacc[1]) + (sacc[2] + sacc[3]);
        cn2[j] = t;
        inv[j] = t > 0.0 ? float(1.0 / t) : 0.f;
        hash[j] = sh[0] + sh[1] + sh[2] + sh[3];
        idx_out[j] = src;
    }
}

template <typename TR>
__global__ __launch_bounds__(256) void k_gather(const u32x4_t* __restrict__ X, const int32_t* __restrict__ idx_in, int b, int nch,
                                                u32x4_t* __restrict__ C, int32_t* __restrict__ idx_out, float* __restrict__ inv,
                                                double* __restrict__ cn2, unsigned long long* __restrict__ hash,
                                                int32_t* __restrict__ eta) {
    gather_row<TR>(X, blockIdx.x, idx_in[blockIdx.x], b, nch, C, idx_out, inv, cn2, hash, eta);
}

// generators j0 .. j0 + gridDim.x - 1, their row numbers in the argument block
template <typename TR>
__global__ __launch_bounds__(256) void k_gather_arg(const u32x4_t* __restrict__ X, const IdxByValue idx_in, int j0, int b, int nch,
                                                    u32x4_t* __restrict__ C, int32_t* __restrict__ idx_out, float* __restrict__ inv,
                                                    double* __restrict__ cn2, unsigned long long* __restrict__ hash,
                                                    int32_t* __restrict__ eta) {
    gather_row<TR>(X, j0 + blockIdx.x, idx_in.v[blockIdx.x], b, nch, C, idx_out, inv, cn2, hash, eta);
}

// ------------------------------------------------------------------------------------------------
// The final word on f(i) and alpha_i.  A token whose leading scores are within 2^-12 (relative) of each other is
// re-decided in fp64: among up to four named candidates (the winner, a non-identical generator that ties with it
// exactly, the runners-up) when every value that close has a name, among all generators otherwise (in the
// workloads here: never seen; three values that close: one token in 250 000).  Such tokens are rare but unevenly
// spread, so a workgroup pools them in an LDS queue (decide_or_queue, called by every lane for its token) and its
// waves then share them out (drain_queue, called by the whole workgroup).
constexpr int kRedoInts = 6;     // row, number of extra candidates (4 = all generators), j1, c1, c2, c3

// Neighbourhood condition (Eq. 2): ||X_i - alpha_i C_f(i)||_2 <= eps ||X_i||_2, i.e. s(i,f(i)) >= (1 - eps^2) ||X_i||^2
// (the residual of a projection: ||X_i||^2 - s).  keep = 1 - eps^2; keep < 0 switches the test off (eps >= 1 can
// drop nothing).  In fp32 the test is trusted outside a band of 2^-11 ||X_i||^2 around the limit; inside it the
// token goes to the fp64 second look, which compares <X_i,C_j>^2 with keep ||X_i||^2 ||C_j||^2 (no division: a row
// that is an exact copy or power-of-two multiple of its generator passes at eps = 0 without rounding).
struct Neighbourhood {
    double keep;           // 1 - eps^2, or negative: no condition
    int* dropped;          // LDS counter of the workgroup
};

// Dot products of one row of X with two generators, in fp64, by the whole wave.  This code runs a handful of times
// per launch, on the critical path of its workgroup: loads go out four chunks per lane at a time (one memory
// latency for rows of up to 256 chunks), and the code is kept small because all of it misses the instruction cache.
template <typename TR>
__device__ __noinline__ void wave_dot2(const u32x4_t* __restrict__ x, const u32x4_t* __restrict__ ca, const u32x4_t* __restrict__ cb,
                                       int nch, double& da, double& db) {
    double acc0 = 0.0, acc1 = 0.0;
    const int lane = threadIdx.x & 63;
#pragma unroll 1
    for (int q0 = 0; q0 < nch; q0 += 4 * kWave) {
        u32x4_t xv[4], av[4], bv[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int q = q0 + t * kWave + lane;
            const uint32_t keep = q < nch ? 0xffffffffu : 0u;       // chunks past the end of the row count as zeros
            const int qq = min(q, nch - 1);
            xv[t] = x[qq] & keep; av[t] = ca[qq]; bv[t] = cb[qq];
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            float a[TR::kPerChunk], b0[TR::kPerChunk], b1[TR::kPerChunk];
            TR::unpack(xv[t], a);
            TR::unpack(av[t], b0);
            TR::unpack(bv[t], b1);
#pragma unroll
            for (int e = 0; e < TR::kPerChunk; ++e) {
                acc0 += double(a[e]) * double(b0[e]);
                acc1 += double(a[e]) * double(b1[e]);
            }
        }
    }
    da = wave_sum(acc0);
    db = wave_sum(acc1);
}

// Called by every lane.  Writes f and alpha of the lane's token unless it needs a second look; then it is queued.
__device__ __forceinline__ void decide_or_queue(const float* __restrict__ inv, const double* __restrict__ cn2,
                                                const unsigned long long* __restrict__ hash, bool valid, int row, const Best& st,
                                                float nx, const Neighbourhood& nb, int32_t* __restrict__ f,
                                                float* __restrict__ alpha, int* q_count, int* q_entries) {
    if (!valid) return;
    bool unsure = false, drop = false;
    if (nb.keep >= 0.0) {
        const float lim = float(nb.keep) * nx, band = 0x1p-11f * nx;
        drop = st.s1 < lim - band;
        unsure = !drop && st.s1 < lim + band;
    }
    int ncand = 0, c1 = 0, c2 = 0, c3 = 0;
    if (st.s1 > 0.f) {
        const float thr = st.s1 * (1.f - 0x1p-12f);
        // an exact tie between two generators whose rows are bit-identical needs no second look: the lower one wins
        if (st.jt >= 0 &&
            !(hash[st.j1] == hash[st.jt] && __double_as_longlong(cn2[st.j1]) == __double_as_longlong(cn2[st.jt])))
            c1 = st.jt, ncand = 1;
        if (st.s2 >= thr) { (ncand == 0 ? c1 : c2) = st.j2; ++ncand; }
        if (st.s3 >= thr) {
            if (st.j3 >= 0) { (ncand == 0 ? c1 : (ncand == 1 ? c2 : c3)) = st.j3; ++ncand; }
            else ncand = 4;
        }
        if (st.s4 >= thr) ncand = 4;
    }
    if (ncand == 0 && !unsure) {
        f[row] = st.j1;
        alpha[row] = drop ? 0.f : st.d1 * inv[st.j1];
        if (drop) atomicAdd(nb.dropped, 1);
    } else {
        int* e = q_entries + atomicAdd(q_count, 1) * kRedoInts;
        e[0] = row; e[1] = ncand; e[2] = st.j1; e[3] = c1; e[4] = c2; e[5] = c3;
    }
}

// Called by the whole workgroup (NWAVES waves) after a barrier that follows the last decide_or_queue.
template <typename TR, int NWAVES>
__device__ __forceinline__ void drain_queue(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ C,
                                            const double* __restrict__ cn2, int nch, int k, const Neighbourhood& nb,
                                            int32_t* __restrict__ f, float* __restrict__ alpha, const int* q_count,
                                            const int* q_entries) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int total = *q_count;
    for (int t = wave; t < total; t += NWAVES) {
        const int* e = q_entries + t * kRedoInts;
        const int row = e[0], rn = e[1];
        const u32x4_t* xr = X + size_t(row) * nch;
        double bs = -1.0, bd = 0.0, bc = 1.0;
        int bj = 0;
        auto take = [&](int j, double d, double c2n) {
            const double sc = c2n > 0.0 ? d * d / c2n : 0.0;
            if (sc > bs) { bs = sc; bd = d; bc = c2n; bj = j; }                   // strict: lowest j keeps a tie
        };
        auto eval2 = [&](int ja, int jb) {                     // ja <= jb; ja == jb evaluates one generator
            const double na = cn2[ja], nb = cn2[jb];          // in flight together with the rows
            double da, db;
            wave_dot2<TR>(xr, C + size_t(ja) * nch, C + size_t(jb) * nch, nch, da, db);
            take(ja, da, na);
            if (jb != ja) take(jb, db, nb);
        };
        if (rn == 0) {
            eval2(e[2], e[2]);             // only the neighbourhood condition is in doubt
        } else if (rn < 4) {
            // the named candidates in increasing j; unused slots sort to the end
            constexpr int kNone = 0x7fffffff;
            int a0 = e[2], a1 = e[3], a2 = rn >= 2 ? e[4] : kNone, a3 = rn >= 3 ? e[5] : kNone;
            auto cx = [](int& x, int& y) { const int lo = min(x, y), hi = max(x, y); x = lo; y = hi; };
            cx(a0, a1); cx(a2, a3); cx(a0, a2); cx(a1, a3); cx(a1, a2);
            eval2(a0, a1);
            if (rn == 2) eval2(a2, a2);
            if (rn == 3) eval2(a2, a3);
        } else {
#pragma unroll 1
            for (int j0 = 0; j0 < k; j0 += 2) eval2(j0, min(j0 + 1, k - 1));
        }
        bool kept = true;
        if (nb.keep >= 0.0) {
            double nx, unused;
            wave_dot2<TR>(xr, xr, xr, nch, nx, unused);
            kept = bd * bd >= nb.keep * nx * bc;
        }
        if (lane == 0) {
            f[row] = bj;
            alpha[row] = (kept && bc > 0.0) ? float(bd / bc) : 0.f;
            if (!kept) atomicAdd(nb.dropped, 1);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// k_score.  Workgroup = NW waves; wave w owns 32*TT tokens; the workgroup owns one column block of
// 32*TG generators.  Roles in the 32x32 MFMA: A operand = generators, B operand = tokens, so a lane
// ends up holding scores of ONE token (lane%32) against 16*TG generators per token fragment.
//
// The hidden dimension is walked in "super-steps" of 8 chunks (128 bytes of a row); an MFMA step u takes
// chunk 4g+u of the window from lane group g, for the token operand and the generator operand alike (the
// order of the hidden index inside a dot product is free, as long as both operands agree).
//
// X: each wave streams its own tokens with fully coalesced loads (8 lanes cover the 128 bytes of one row and
// super-step), D-1 super-steps ahead in registers, then passes them through a wave-private LDS tile to reach
// the MFMA layout (lane r needs 16 bytes of row r).  Inside the tile, row r keeps chunk c at position c^(r&7),
// which makes both the lane-linear writes and the column reads free of bank conflicts.
// C: staged through LDS in stages of 64/TG chunks per generator (32 KiB per stage), double buffered; the
// global loads of the next one or two stages are in flight in registers while a stage is consumed.
// The generator fragments of a super-step are read from LDS one group of up to four ahead of their MFMAs, and the
// loads, stashes and stage stores of the super-step are placed between those groups.
// FUSED (one column block holds every generator): the epilogue takes the final decision itself and writes f and
// alpha; otherwise it writes one candidate record per token and column block for k_finalize.
template <typename TR, int TG, int TT, int NW, bool ALIGNED, bool FUSED>
__global__ __launch_bounds__(64 * NW) void k_score(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ C,
                                                   const float* __restrict__ inv, const double* __restrict__ cn2,
                                                   const unsigned long long* __restrict__ hash, int b, int nch, int k, int ncb,
                                                   u32x4_t* __restrict__ cand, int32_t* __restrict__ f, float* __restrict__ alpha,
                                                   double keep, int32_t* __restrict__ eta) {
    constexpr int NT = 64 * NW;
    const bool want_norm = keep >= 0.0;           // a finite tolerance: ||X_i||^2 is needed (uniform over the grid)
    constexpr int GB = 32 * TG;          // generators per column block
    constexpr int SS = 8 / TG;           // super-steps per stage
    constexpr int CPS = 8 * SS;          // chunks per generator per stage
    constexpr int RS = CPS + 1;          // LDS row stride in chunks (odd: conflict-free 16-byte reads down a column)
    constexpr int CLOADS = GB * CPS / NT;   // chunks of C per thread per stage
    constexpr int CBUF = GB * RS;        // chunks per C buffer
    constexpr int XSLOT = TT * 256;      // chunks per X slot (TT fragments of 32 rows x 8 chunks)
    constexpr int D = TG == 8 ? 3 : 4;   // X ring depth in registers (super-steps); 128 accumulator registers leave room for 3
    constexpr int UN = SS > D ? SS : D;  // super-steps per unrolled body: a multiple of SS and of D
    // Stages of C in flight in registers, PD of them.  Short stages (one or two super-steps) are over before a load
    // from L2 has come back, so two are in flight where the registers allow; the register slot of a stage is its
    // parity, which is static when the unrolled body holds an even number of stages.
    constexpr int PD = (UN / SS) % 2 == 0 ? 2 : 1;
    static_assert(GB * CPS % NT == 0, "stage does not divide over the threads");

    __shared__ u32x4_t lds_raw[2 * CBUF + NW * 2 * XSLOT];
    __shared__ __attribute__((aligned(16))) float lds_inv[GB];
    __shared__ int redo_count, drop_count;
    __shared__ int redo_entries[FUSED ? 32 * TT * NW * kRedoInts : 1];   // every token of the tile could need a second look
    u32x4_t* const lds_c = lds_raw;                                         // [2][CBUF]
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, r = lane & 31, g = lane >> 5;
    u32x4_t* const lds_x = lds_raw + 2 * CBUF + wave * (2 * XSLOT);         // [2][XSLOT], private to this wave
    // Workgroups are handed to the 8 XCDs round-robin and every XCD has its own L2.  With several column blocks the
    // workgroups of one row tile (which stream the same rows of X) take consecutive places in the sequence of ONE XCD,
    // so that X comes from HBM once and from that L2 for the other column blocks.
    int cb = 0, rt = blockIdx.x;
    if (ncb > 1) {
        const int xcd = blockIdx.x % 8, q = blockIdx.x / 8;
        cb = q % ncb;
        rt = (q / ncb) * 8 + xcd;
        if (rt * (32 * TT * NW) >= b) return;          // the grid is rounded up to whole groups of 8 row tiles
    }
    const int gen0 = cb * GB;

    if (tid == 0) { redo_count = 0; drop_count = 0; }          // published by the barriers of the main loop
    for (int t = tid; t < GB; t += NT) {
        const int j = gen0 + t;
        lds_inv[t] = j < k ? inv[j] : -1.f;        // negative marks a slot past the last generator
    }

    // coalesced view of this wave's tokens: load i of fragment tt covers rows 8i .. 8i+7, lane L the row 8i + L/8
    // and the chunk (L%8) ^ (L/8) of the window, so that it lands at position L%8 of its row in the tile
    const int row_base = rt * (32 * TT * NW) + wave * (32 * TT);
    const int xchunk = (lane & 7) ^ (lane >> 3);
    const u32x4_t* xrow[TT][4];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int row = row_base + 32 * tt + 8 * i + (lane >> 3);
            row = row < b ? row : b - 1;           // rows past the end are computed on a valid row and never stored
            xrow[tt][i] = X + size_t(row) * nch;
        }

    f32x16_t acc[TG][TT];
    float nrm[TT][4];                              // this lane's share of ||X_i||^2 for the four rows it loads
#pragma unroll
    for (int t = 0; t < TT; ++t) {
#pragma unroll
        for (int a = 0; a < TG; ++a)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][t][i] = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) nrm[t][i] = 0.f;
    }

    const int nstages = (nch + CPS - 1) / CPS;
    const int nss = (nch + 7) / 8;               // super-steps
    // Every workgroup walks the hidden dimension from a different starting window and wraps around (a dot product
    // does not care where it starts).  Without this all workgroups sit at the same column of their rows at the same
    // time, and since rows are a power of two apart the whole chip then leans on a few memory channels.
    // With several column blocks the workgroups of one XCD walk in step instead (one starting window per XCD): between
    // them they then hold one window of all of C and of their rows of X in that XCD's L2 at a time, each line fetched
    // once and hit by the others; walking apart, every workgroup's pass over its block of C missed the L2.
    const int rot = ncb > 1 ? int(blockIdx.x % 8) * (nss / 8) % nss : (rt * 5) % nss;
    auto turned = [&](int v) {                   // walk position -> window of the row; positions past the end repeat the last
        const int a = min(v, nss - 1) + rot;
        return a >= nss ? a - nss : a;
    };

    u32x4_t creg[PD][CLOADS];
    auto load_c = [&](int stage, int slot) {      // stages past the last one re-read the last window (never stored)
#pragma unroll
        for (int i = 0; i < CLOADS; ++i) {
            const int q = tid + NT * i;
            const int row = q / CPS, cc = q % CPS;
            const int j = gen0 + row, c = turned(stage * SS + cc / 8) * 8 + (cc & 7);
            // Clamped addresses, no guard and no mask: a guarded load costs a branch per chunk, and a mask makes
            // the compiler wait for the load where it is issued.  Rows past the last generator are ignored by
            // the epilogue; chunks past the end of a row meet zero chunks of X.
            creg[slot][i] = C[size_t(min(j, k - 1)) * nch + min(c, nch - 1)];
        }
    };
    auto store_c = [&](int buf, int slot) {
#pragma unroll
        for (int i = 0; i < CLOADS; ++i) {
            const int q = tid + NT * i;
            lds_c[buf * CBUF + (q / CPS) * RS + (q % CPS)] = creg[slot][i];
        }
    };
    u32x4_t xr[D][TT][4];
    auto load_x = [&](u32x4_t (&dst)[TT][4], int sstep) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (ALIGNED) {        // rows are whole super-steps: clamp the super-step, nothing to mask
                    dst[tt][i] = xrow[tt][i][turned(sstep) * 8 + xchunk];
                } else {
                    const int c = turned(sstep) * 8 + xchunk;
                    const uint32_t keep = c < nch ? 0xffffffffu : 0u;
                    dst[tt][i] = xrow[tt][i][min(c, nch - 1)] & keep;
                }
            }
    };
    // registers -> this wave's LDS tile; `fresh` (uniform): the window has not been stashed before, so with a finite
    // tolerance its squares are added to the row norms (every chunk of X passes here exactly once)
    auto stash_x = [&](const u32x4_t (&src)[TT][4], int slot, bool fresh) {
        const uint32_t live = fresh ? 0xffffffffu : 0u;      // windows past the end of the walk enter as zeros
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int i = 0; i < 4; ++i) lds_x[slot * XSLOT + tt * 256 + i * 64 + lane] = src[tt][i] & live;
        if (want_norm && fresh) {
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float e[TR::kPerChunk];
                    TR::unpack(src[tt][i], e);
#pragma unroll
                    for (int q = 0; q < TR::kPerChunk; ++q) nrm[tt][i] = fmaf(e[q], e[q], nrm[tt][i]);
                }
        }
    };

    load_c(0, 0);
#pragma unroll
    for (int d = 0; d < D - 1; ++d) load_x(xr[d], d);
    store_c(0, 0);
#pragma unroll
    for (int d = 1; d <= PD; ++d) load_c(d, d % PD);        // stage d travels in register slot d % PD
    stash_x(xr[0], 0, true);
    __syncthreads();

    const int nbody = (nss + UN - 1) / UN;
    int buf = 0, stage = 0;
    for (int bi = 0; bi < nbody; ++bi) {
#pragma unroll
        for (int p = 0; p < UN; ++p) {
            const int gs = bi * UN + p;                      // super-step
            if (p % SS == 0) stage = gs / SS;                // a stage of C begins
            // What a super-step does besides its MFMAs, in three parts that are placed between the MFMA groups so that
            // their issue slots and waits hide behind matrix work (a wave issues in order; an MFMA keeps the matrix
            // pipe busy for 32 cycles during which the wave's next instructions of other kinds go out):
            auto side = [&](int part) {
                if (part == 0) load_x(xr[(p + D - 1) % D], gs + D - 1);
                if (part == 1) stash_x(xr[(p + 1) % D], (gs + 1) & 1, gs + 1 < nss);   // next super-step's tokens, other slot
                if (part == 2 && p % SS == SS - 1) {         // the stage ends: fill the C buffer nobody reads now
                    // (also past the last stage, with the last window again: the MFMAs of the tail multiply what
                    // this buffer holds by zeros, so it must hold finite numbers)
                    store_c(buf ^ 1, (p / SS + 1) % PD);
                    // the slot is free again: the loads of stage + 1 + PD have the barrier and PD whole stages to
                    // come back (issued on every path, so that waits stay counted, not full)
                    load_c(stage + 1 + PD, (p / SS + 1) % PD);
                }
            };
            constexpr bool RIDE = TG < 8;       // with 128 accumulator registers the longer live ranges would spill
            if (!RIDE) { side(0); side(1); side(2); }
            {   // (in the tail of the last body the walk is over: its windows were stashed as zeros and add nothing)
                const u32x4_t* cbuf = lds_c + buf * CBUF;
                const u32x4_t* xbuf = lds_x + (gs & 1) * XSLOT;
                // The 4 TG generator fragments of the super-step (MFMA step u, fragment tg: number u TG + tg) are
                // taken in groups of at most four.  The LDS reads of group q+1 are issued before the MFMAs of group q,
                // and the scheduling barriers keep that order: left alone, the compiler pulls every read down to its
                // MFMA to save registers and each MFMA then waits out a full LDS latency.
                constexpr int GRP = TG < 4 ? TG : 4, NGRP = 4 * TG / GRP;
                constexpr int S1 = NGRP / 4 > 1 ? NGRP / 4 : 1, S2 = NGRP / 2 > 2 ? NGRP / 2 : 2;   // groups the parts follow
                u32x4_t a[2][GRP], bx[2][TT];
                auto fetch_a = [&](int grp, int which) {
#pragma unroll
                    for (int i = 0; i < GRP; ++i) {
                        const int t = grp * GRP + i, u = t / TG, tg = t % TG;
                        a[which][i] = cbuf[(32 * tg + r) * RS + (p % SS) * 8 + 4 * g + u];
                    }
                };
                auto fetch_b = [&](int u, int which) {
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) bx[which][tt] = xbuf[tt * 256 + r * 8 + ((4 * g + u) ^ (r & 7))];
                };
                fetch_b(0, 0);
                fetch_a(0, 0);
#pragma unroll
                for (int grp = 0; grp < NGRP; ++grp) {
                    const int u = grp * GRP / TG;
                    if (grp + 1 < NGRP) {
                        const int un = (grp + 1) * GRP / TG;
                        if (un != u) fetch_b(un, un & 1);
                        fetch_a(grp + 1, (grp + 1) & 1);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < GRP; ++i)
#pragma unroll
                        for (int tt = 0; tt < TT; ++tt) TR::mma(a[grp & 1][i], bx[u & 1][tt], acc[(grp * GRP + i) % TG][tt]);
                    if (RIDE && grp == 0) side(0);
                    if (RIDE && grp == S1) side(1);
                    if (RIDE && grp == S2) side(2);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (p % SS == SS - 1) {                          // the stage ends: publish the next one
                __syncthreads();
                buf ^= 1;
            } else {
                wave_lds_sync();                             // the stashed tokens are read by other lanes of this wave
            }
        }
    }

    // Epilogue.  D layout of the 32x32 MFMA: register i of lane (r,g) is generator 8*(i/4)+4*g+(i%4), token r.
    // The scores go through LDS (all tiles are free after the last barrier) so that the scan over generators
    // is a small rolled loop instead of hundreds of unrolled compare/select chains: each pass dumps PG
    // generators x 32 tokens per wave, then lane (r,g) scans half of them for token r in increasing order.
    constexpr int PFMAX = NW == 8 ? 2 : 4;
    constexpr int PF = TG < PFMAX ? TG : PFMAX;   // fragments per pass
    constexpr int PG = 32 * PF;              // generators per pass
    constexpr int SROW = PG + 4;             // floats per token row (padding: conflict-free 16-byte accesses)
    static_assert(NW * 32 * SROW * sizeof(float) <= sizeof(lds_raw), "score dump does not fit");
    float* sdump = reinterpret_cast<float*>(lds_raw) + wave * (32 * SROW);
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        auto dump = [&](int h) {                 // scores of pass h -> this wave's LDS tile, [token][generator]
#pragma unroll
            for (int pf = 0; pf < PF; ++pf)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x16_t& v = acc[h * PF + pf][tt];
                    *reinterpret_cast<float4*>(&sdump[r * SROW + 32 * pf + 8 * q + 4 * g]) =
                        make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
                }
            wave_lds_sync();
        };
        const float* srow = &sdump[r * SROW + g * (PG / 2)];

        // Per lane, over its half of every pass: the largest score m1 (lowest j on ties) with its dot product, the
        // lowest other generator reaching m1 exactly (jt), the largest score strictly below m1 (m2, lowest j: j2)
        // and the largest strictly below m2 (m3, value only).
        float m1 = -1.f, m2 = -2.f, m3 = -3.f, dm = 0.f;
        int jm = 0, jt = -1, j2 = 0;
#pragma unroll
        for (int h = 0; h < TG / PF; ++h) {
            dump(h);
            const int jl0 = h * PG + g * (PG / 2);
#pragma unroll 2
            for (int c = 0; c < PG / 2; c += 4) {
                const float4 d4 = *reinterpret_cast<const float4*>(&srow[c]);
                const float4 iv4 = *reinterpret_cast<const float4*>(&lds_inv[jl0 + c]);
                const float dd[4] = {d4.x, d4.y, d4.z, d4.w}, iv[4] = {iv4.x, iv4.y, iv4.z, iv4.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float sc = iv[e] >= 0.f ? dd[e] * dd[e] * iv[e] : -3.f;      // slots past the last generator
                    const int j = gen0 + jl0 + c + e;
                    const bool up = sc > m1, tie = sc == m1;
                    const bool mid = !up && !tie && sc > m2;
                    const bool low = sc < m2 && sc > m3;
                    m3 = (up || mid) ? m2 : (low ? sc : m3);
                    j2 = up ? jm : (mid ? j : j2);
                    m2 = up ? m1 : (mid ? sc : m2);
                    jt = up ? -1 : ((tie && jt < 0) ? j : jt);
                    dm = up ? dd[e] : dm;
                    jm = up ? j : jm;
                    m1 = up ? sc : m1;
                }
            }
            wave_lds_sync();
        }
        Best best;
        best.init();
        best.s1 = m1; best.j1 = jm; best.d1 = dm; best.jt = jt; best.s2 = m2; best.j2 = j2; best.s3 = m3;
        // Second pass, in the rare wave where some lane has three distinct values within 2^-12 of each other: list who
        // attains the values that close to the lane's maximum (only those can matter to the final decision).
        const bool crowded = m1 > 0.f && m3 >= m1 * (1.f - 0x1p-12f);
        if (__builtin_amdgcn_ballot_w64(crowded) != 0ull) {
            const float thr = m1 * (1.f - 0x1p-12f);
            best.s2 = -2.f; best.j2 = 0; best.s3 = -3.f; best.j3 = -1; best.s4 = -4.f;
            if (!crowded) { best.s2 = m2; best.j2 = j2; best.s3 = m3; }
#pragma unroll
            for (int h = 0; h < TG / PF; ++h) {
                dump(h);
                const int jl0 = h * PG + g * (PG / 2);
#pragma unroll 2
                for (int c = 0; c < PG / 2; c += 4) {
                    const float4 d4 = *reinterpret_cast<const float4*>(&srow[c]);
                    const float4 iv4 = *reinterpret_cast<const float4*>(&lds_inv[jl0 + c]);
                    const float dd[4] = {d4.x, d4.y, d4.z, d4.w}, iv[4] = {iv4.x, iv4.y, iv4.z, iv4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float sc = iv[e] >= 0.f ? dd[e] * dd[e] * iv[e] : -3.f;
                        const bool hit = crowded && sc >= thr && sc < m1;
                        if (__builtin_amdgcn_ballot_w64(hit) != 0ull) {
                            if (hit) best.insert_lower(sc, gen0 + jl0 + c + e);
                        }
                    }
                }
                wave_lds_sync();
            }
        }
        // the two lanes of a token join their halves
        {
            Best o;
            o.s1 = __shfl_xor(best.s1, 32); o.j1 = __shfl_xor(best.j1, 32); o.d1 = __shfl_xor(best.d1, 32);
            o.jt = __shfl_xor(best.jt, 32); o.s2 = __shfl_xor(best.s2, 32); o.j2 = __shfl_xor(best.j2, 32);
            o.s3 = __shfl_xor(best.s3, 32); o.j3 = __shfl_xor(best.j3, 32); o.s4 = __shfl_xor(best.s4, 32);
            best.merge(o);
        }
        const int row = row_base + 32 * tt + r;
        // ||X_i||^2: row 8 i + L/8 of the fragment was loaded by the eight lanes L/8 = const, as their load i
        float nx = 0.f;
        if (want_norm) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float v = nrm[tt][i];
                v += __shfl_xor(v, 1); v += __shfl_xor(v, 2); v += __shfl_xor(v, 4);
                const float w = __shfl(v, (r & 7) * 8);
                nx = (i == (r >> 3)) ? w : nx;
            }
        }
        const Neighbourhood nb{keep, &drop_count};
        if (FUSED) {
            // (one column block: generator j's 1/||C_j||^2 sits in lds_inv[j], no need to go to memory for it)
            decide_or_queue(lds_inv, cn2, hash, g == 0 && row < b, row, best, nx, nb, f, alpha, &redo_count, redo_entries);
        } else {
            if (g == 0 && row < b) {
                u32x4_t* rec = cand + (size_t(row) * ncb + cb) * 2;
                best.store(rec);
                Best::store_norm(rec, nx);
            }
        }
    }
    if (FUSED) {
        const Neighbourhood nb{keep, &drop_count};
        __syncthreads();
        drain_queue<TR, NW>(X, C, cn2, nch, k, nb, f, alpha, &redo_count, redo_entries);
        if (want_norm) {
            __syncthreads();
            if (tid == 0 && drop_count > 0) atomicAdd(eta, drop_count);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// k_finalize: one thread per token; only needed when the generators span several column blocks.
template <typename TR>
__global__ __launch_bounds__(256) void k_finalize(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ C,
                                                  const float* __restrict__ inv, const double* __restrict__ cn2,
                                                  const unsigned long long* __restrict__ hash,
                                                  const u32x4_t* __restrict__ cand, int b, int nch, int k, int ncb,
                                                  int32_t* __restrict__ f, float* __restrict__ alpha, double keep,
                                                  int32_t* __restrict__ eta) {
    const int row = blockIdx.x * 256 + threadIdx.x;
    const bool valid = row < b;
    Best st;
    st.init();
    if (valid) {
        for (int cb = 0; cb < ncb; ++cb) {
            Best o;
            o.load(cand + (size_t(row) * ncb + cb) * 2);
            if (cb == 0) st = o; else st.merge(o);
        }
    }
    __shared__ int redo_count, drop_count;
    __shared__ int redo_entries[256 * kRedoInts];
    if (threadIdx.x == 0) { redo_count = 0; drop_count = 0; }
    __syncthreads();
    const Neighbourhood nb{keep, &drop_count};
    const float nx = (valid && keep >= 0.0) ? Best::load_norm(cand + size_t(row) * ncb * 2) : 0.f;    // every block stores the same value
    decide_or_queue(inv, cn2, hash, valid, row, st, nx, nb, f, alpha, &redo_count, redo_entries);
    __syncthreads();
    drain_queue<TR, 4>(X, C, cn2, nch, k, nb, f, alpha, &redo_count, redo_entries);
    if (keep >= 0.0) {
        __syncthreads();
        if (threadIdx.x == 0 && drop_count > 0) atomicAdd(eta, drop_count);
    }
}

// ------------------------------------------------------------------------------------------------ host side

struct ScoreArgs {
    const void* X; const void* C; const float* inv; const double* cn2; const unsigned long long* hash;
    int b, nch, k;
    u32x4_t* cand; int32_t* f; float* alpha;
    double keep; int32_t* eta;
};

template <typename TR, int TG, int TT, int NW, bool FUSED>
static void launch_score_cfg(const CompressPlan& pl, const ScoreArgs& a, hipStream_t s) {
    dim3 grid((unsigned)(pl.ncb > 1 ? (pl.row_tiles + 7) / 8 * 8 * pl.ncb : pl.row_tiles));
    if (a.nch % 8 == 0)      // every row is a whole number of 128-byte super-steps
        hipLaunchKernelGGL((k_score<TR, TG, TT, NW, true, FUSED>), grid, dim3(64 * NW), 0, s, (const u32x4_t*)a.X,
                           (const u32x4_t*)a.C, a.inv, a.cn2, a.hash, a.b, a.nch, a.k, pl.ncb, a.cand, a.f, a.alpha, a.keep, a.eta);
    else
        hipLaunchKernelGGL((k_score<TR, TG, TT, NW, false, FUSED>), grid, dim3(64 * NW), 0, s, (const u32x4_t*)a.X,
                           (const u32x4_t*)a.C, a.inv, a.cn2, a.hash, a.b, a.nch, a.k, pl.ncb, a.cand, a.f, a.alpha, a.keep, a.eta);
}

template <typename TR, int TG, bool FUSED>
static void launch_score_tg(const CompressPlan& pl, const ScoreArgs& a, hipStream_t s) {
    if (pl.nw == 8) launch_score_cfg<TR, TG, 1, 8, FUSED>(pl, a, s);
    else if (pl.nw == 4) launch_score_cfg<TR, TG, 1, 4, FUSED>(pl, a, s);
    else launch_score_cfg<TR, TG, 1, 2, FUSED>(pl, a, s);
}

// One column block: the fused kernel.  Several column blocks: one record per token and block for k_finalize.
template <typename TR, bool FUSED>
static void launch_score_blocks(const CompressPlan& pl, const ScoreArgs& a, hipStream_t s) {
    switch (pl.tg) {
        case 1: launch_score_tg<TR, 1, FUSED>(pl, a, s); break;
        case 2: launch_score_tg<TR, 2, FUSED>(pl, a, s); break;
        case 4: launch_score_tg<TR, 4, FUSED>(pl, a, s); break;
        default: launch_score_tg<TR, 8, FUSED>(pl, a, s); break;
    }
}

template <typename TR>
static void launch_score(const CompressPlan& pl, const ScoreArgs& a, hipStream_t s) {
    if (pl.ncb > 1) launch_score_blocks<TR, false>(pl, a, s);
    else launch_score_blocks<TR, true>(pl, a, s);
}

// idx_dev: the generators' row numbers in device memory, or NULL: then idx_host holds them (host memory, only read
// during the call) and they travel in argument blocks.
template <typename TR>
static pamm_status run_compress(const CompressPlan& pl, const void* X, int b, int n, int k, const int32_t* idx_dev,
                                const int32_t* idx_host, double keep, void* C, int32_t* f, float* alpha, int32_t* eta, char* ws,
                                hipStream_t s) {
    const int nch = n / TR::kPerChunk;
    int32_t* idx = reinterpret_cast<int32_t*>(ws + pl.off_idx);
    float* inv = reinterpret_cast<float*>(ws + pl.off_inv);
    double* cn2 = reinterpret_cast<double*>(ws + pl.off_cn2);
    unsigned long long* hash = reinterpret_cast<unsigned long long*>(ws + pl.off_hash);
    u32x4_t* cand = reinterpret_cast<u32x4_t*>(ws + pl.off_cand);

    {
        ScopedSpan span(kGather, s);
        if (idx_dev) {
            hipLaunchKernelGGL((k_gather<TR>), dim3(k), dim3(256), 0, s, (const u32x4_t*)X, idx_dev, b, nch, (u32x4_t*)C, idx, inv, cn2,
                               hash, eta);
        } else {
            for (int j0 = 0; j0 < k; j0 += kArgGenerators) {
                const int cnt = k - j0 < kArgGenerators ? k - j0 : kArgGenerators;
                IdxByValue ia;
                for (int j = 0; j < kArgGenerators; ++j) ia.v[j] = j < cnt ? idx_host[j0 + j] : 0;
                hipLaunchKernelGGL((k_gather_arg<TR>), dim3(cnt), dim3(256), 0, s, (const u32x4_t*)X, ia, j0, b, nch, (u32x4_t*)C, idx,
                                   inv, cn2, hash, eta);
            }
        }
    }
    {
        ScopedSpan span(kScore, s);
        launch_score<TR>(pl, ScoreArgs{X, C, inv, cn2, hash, b, nch, k, cand, f, alpha, keep, eta}, s);
    }
    if (pl.ncb > 1) {
        ScopedSpan span(kFinalize, s);
        hipLaunchKernelGGL((k_finalize<TR>), dim3((b + 255) / 256), dim3(256), 0, s, (const u32x4_t*)X, (const u32x4_t*)C, inv, cn2,
                           hash, cand, b, nch, k, pl.ncb, f, alpha, keep, eta);
    }
    return hipGetLastError() == hipSuccess ? PAMM_OK : PAMM_ERR_DEVICE;
}

}  // namespace pamm

using namespace pamm;

static pamm_status compress_idx_impl(const void* X, int64_t b, int64_t n, int64_t k, const int32_t* idx_dev, double keep,
                                     pamm_dtype dt, void* C, int32_t* f, float* alpha, int32_t* eta, void* ws, size_t ws_bytes,
                                     void* stream) {
    CompressPlan pl;
    pamm_status st = check_compress_args(X, b, n, k, dt, C, f, alpha, ws, ws_bytes, &pl);
    if (st != PAMM_OK) return st;
    if (!idx_dev) return PAMM_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (dt == PAMM_BF16)
        return run_compress<Bf16>(pl, X, int(b), int(n), int(k), idx_dev, nullptr, keep, C, f, alpha, eta, (char*)ws, s);
    return run_compress<F32>(pl, X, int(b), int(n), int(k), idx_dev, nullptr, keep, C, f, alpha, eta, (char*)ws, s);
}

static pamm_status compress_seed_impl(const void* X, int64_t b, int64_t n, int64_t k, uint64_t seed, double keep, pamm_dtype dt,
                                      void* C, int32_t* f, float* alpha, int32_t* eta, void* ws, size_t ws_bytes, void* stream) {
    CompressPlan pl;
    pamm_status st = check_compress_args(X, b, n, k, dt, C, f, alpha, ws, ws_bytes, &pl);
    if (st != PAMM_OK) return st;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);

    // the sampled row numbers travel in the gather kernels' argument blocks
    int32_t idx_host[kMaxGenerators];
    st = pamm_sample_indices(b, k, seed, idx_host);
    if (st != PAMM_OK) return st;
    if (dt == PAMM_BF16)
        return run_compress<Bf16>(pl, X, int(b), int(n), int(k), nullptr, idx_host, keep, C, f, alpha, eta, (char*)ws, s);
    return run_compress<F32>(pl, X, int(b), int(n), int(k), nullptr, idx_host, keep, C, f, alpha, eta, (char*)ws, s);
}

extern "C" pamm_status pamm_compress_idx(const void* X, int64_t b, int64_t n, int64_t k, const int32_t* idx_dev, pamm_dtype dt,
                                         void* C, int32_t* f, float* alpha, void* ws, size_t ws_bytes, void* stream) {
    return compress_idx_impl(X, b, n, k, idx_dev, -1.0, dt, C, f, alpha, nullptr, ws, ws_bytes, stream);
}

extern "C" pamm_status pamm_compress(const void* X, int64_t b, int64_t n, int64_t k, uint64_t seed, pamm_dtype dt, void* C,
                                     int32_t* f, float* alpha, void* ws, size_t ws_bytes, void* stream) {
    return compress_seed_impl(X, b, n, k, seed, -1.0, dt, C, f, alpha, nullptr, ws, ws_bytes, stream);
}

extern "C" pamm_status pamm_compress_idx_eps(const void* X, int64_t b, int64_t n, int64_t k, const int32_t* idx_dev, float eps,
                                             pamm_dtype dt, void* C, int32_t* f, float* alpha, int32_t* eta, void* ws,
                                             size_t ws_bytes, void* stream) {
    double keep;
    if (!eta || !aligned4(eta) || keep_of(eps, &keep) != PAMM_OK) return PAMM_ERR_INVALID_ARG;
    return compress_idx_impl(X, b, n, k, idx_dev, keep, dt, C, f, alpha, eta, ws, ws_bytes, stream);
}

extern "C" pamm_status pamm_compress_eps(const void* X, int64_t b, int64_t n, int64_t k, uint64_t seed, float eps, pamm_dtype dt,
                                         void* C, int32_t* f, float* alpha, int32_t* eta, void* ws, size_t ws_bytes, void* stream) {
    double keep;
    if (!eta || !aligned4(eta) || keep_of(eps, &keep) != PAMM_OK) return PAMM_ERR_INVALID_ARG;
    return compress_seed_impl(X, b, n, k, seed, keep, dt, C, f, alpha, eta, ws, ws_bytes, stream);
}
