// pamm_compress / pamm_compress_idx and their _eps forms: Alg. 1, procedure Compress.  With a finite tolerance
// (Eq. 2) the score kernel also sums ||X_i||^2 from the chunks of X as they pass through its registers, and the
// final decision drops the rows whose best representative is outside the neighbourhood.
//
// Launches on the caller's stream:
//   k_gather    C_j = X[idx_j] (bit copy), ||C_j||^2 in fp64, a content hash per generator (k_gather_arg: the same
//               with up to 512 sampled row numbers in the kernel's argument block)
//   k_dedupe    only with more than 256 generators: 1/||C_j|| per generator, 0 for those that can never win (zero
//               rows, and bit-identical copies of a lower-numbered generator: lowest j wins a tie by definition)
//   k_score     streams X once; D = C X^T on the matrix cores with C staged through LDS, then per token the largest
//               and second largest |<X_i,C_j>| / ||C_j|| (the square root of the score of Lemma 1) straight from the
//               accumulator registers.  With up to 256 generators (one column block) it also takes the final
//               decision: f, alpha (Eq. 1), the few rows whose leading scores are too close for fp32 to separate
//               being re-decided in fp64 by the wave that owns them
//   k_finalize  only with more than 256 generators: merges the column blocks and takes that final decision
#include <hip/hip_runtime.h>

#include "pamm_device.h"
#include "pamm_plan.h"
#include "pamm_profile.h"

namespace pamm {

// ------------------------------------------------------------------------------------------------
// What the score kernel keeps of a token after its pass over one column block.  With r(i,j) = |<X_i,C_j>| / ||C_j||
// (r^2 is the score <X_i,C_j>^2 / ||C_j||^2 of Lemma 1, so both have the same argmax):
//   m1   the largest r over the block's generators,  j1 the lowest generator attaining it,
//   a1   <X_i,C_j1> / ||C_j1|| with its sign (alpha_i = a1 / ||C_j1||, Eq. 1),
//   m2   the second largest r (equal to m1 when two generators attain it).
// Generators that can never win are left out by giving them the factor 1/||C_j|| = 0: zero rows, and bit-identical
// copies of a lower-numbered generator (padding tokens sampled twice; the lowest j wins a tie by definition).
// A token whose m2 is within kBand (relative) of m1 cannot be decided in fp32: the generators within the band are
// named (up to kMaxNamed of them) and the decision among them is taken again in fp64.
constexpr int kMaxNamed = 6;              // named candidates per token and column block
constexpr int kTooMany = kMaxNamed + 1;   // more than that: every generator is evaluated again
constexpr float kBand = 0x1.2p-13f;       // on r; about 2^-12 on the score r^2

// 32-byte record per token and column block (several column blocks only): generator numbers fit 16 bits (k <= 16384)
struct BlockRecord {
    float m1, a1;
    int j1, cnt;                 // cnt: 0 = nobody else within the band, 1..kMaxNamed = names[] (j1 among them), kTooMany
    int names[kMaxNamed];

    __device__ __forceinline__ void store(u32x4_t* dst, float nx) const {
        dst[0] = u32x4_t{__float_as_uint(m1), __float_as_uint(a1), uint32_t(j1) | (uint32_t(cnt) << 16),
                         uint32_t(names[0]) | (uint32_t(names[1]) << 16)};
        dst[1] = u32x4_t{uint32_t(names[2]) | (uint32_t(names[3]) << 16), uint32_t(names[4]) | (uint32_t(names[5]) << 16),
                         __float_as_uint(nx), 0u};
    }
    __device__ __forceinline__ void load_lead(const u32x4_t* src) {
        const u32x4_t p = src[0];
        m1 = __uint_as_float(p.x); a1 = __uint_as_float(p.y); j1 = int(p.z & 0xffffu); cnt = int(p.z >> 16);
        names[0] = int(p.w & 0xffffu); names[1] = int(p.w >> 16);
    }
    __device__ __forceinline__ void load_rest(const u32x4_t* src) {
        const u32x4_t q = src[1];
        names[2] = int(q.x & 0xffffu); names[3] = int(q.x >> 16); names[4] = int(q.y & 0xffffu); names[5] = int(q.y >> 16);
    }
    static __device__ __forceinline__ float load_norm(const u32x4_t* src) { return __uint_as_float(src[1].z); }
};

// ------------------------------------------------------------------------------------------------
// k_gather: one workgroup per generator.  The row numbers come from memory (caller-chosen generators) or ride in the
// kernel's own argument block, kArgGenerators per launch (k_gather_arg): sampled indices then need no buffer that
// outlives the call, and a captured launch replays with the indices it was captured with.
constexpr int kArgGenerators = 512;
struct IdxByValue { int32_t v[kArgGenerators]; };

template <typename TR>
__device__ __forceinline__ void gather_row(const u32x4_t* __restrict__ X, int j, int src, int b, int nch, u32x4_t* __restrict__ C,
                                           int32_t* __restrict__ idx_out, float* __restrict__ rn, double* __restrict__ cn2,
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
        rn[j] = t > 0.0 ? float(1.0 / sqrt(t)) : 0.f;      // 1/||C_j||; a zero row can never win (copies: see k_dedupe)
        hash[j] = sh[0] + sh[1] + sh[2] + sh[3];
        idx_out[j] = src;
    }
}

template <typename TR>
__global__ __launch_bounds__(256) void k_gather(const u32x4_t* __restrict__ X, const int32_t* __restrict__ idx_in, int b, int nch,
                                                u32x4_t* __restrict__ C, int32_t* __restrict__ idx_out, float* __restrict__ rn,
                                                double* __restrict__ cn2, unsigned long long* __restrict__ hash,
                                                int32_t* __restrict__ eta) {
    gather_row<TR>(X, blockIdx.x, idx_in[blockIdx.x], b, nch, C, idx_out, rn, cn2, hash, eta);
}

// generators j0 .. j0 + gridDim.x - 1, their row numbers in the argument block
template <typename TR>
__global__ __launch_bounds__(256) void k_gather_arg(const u32x4_t* __restrict__ X, const IdxByValue idx_in, int j0, int b, int nch,
                                                    u32x4_t* __restrict__ C, int32_t* __restrict__ idx_out, float* __restrict__ rn,
                                                    double* __restrict__ cn2, unsigned long long* __restrict__ hash,
                                                    int32_t* __restrict__ eta) {
    gather_row<TR>(X, j0 + blockIdx.x, idx_in.v[blockIdx.x], b, nch, C, idx_out, rn, cn2, hash, eta);
}

// ------------------------------------------------------------------------------------------------
// k_dedupe: for the shapes with several column blocks (with one block the score kernel does this itself), rn[j] <- 0
// for every generator whose row is a bit-identical copy of a lower-numbered one (same content hash, same fp64 norm):
// it can never win, lowest j takes a tie.  64 generators per workgroup, four threads each, which share the
// comparisons with the lower-numbered generators; their (hash, norm) pairs pass through LDS 2048 at a time, all
// loads of a pass issued together (the kernel is a chain of memory latencies, not of work).
__global__ __launch_bounds__(256) void k_dedupe(const double* __restrict__ cn2, const unsigned long long* __restrict__ hash, int k,
                                                float* __restrict__ rn) {
    typedef __attribute__((ext_vector_type(2))) unsigned long long u64x2_t;
    constexpr int TILE = 2048, PER = TILE / 256;
    __shared__ u64x2_t tile[TILE];
    __shared__ int copy_of_lower[64];
    const int tid = threadIdx.x, part = tid >> 6;
    const int j = blockIdx.x * 64 + (tid & 63), jj = min(j, k - 1);
    const u64x2_t mine = {hash[jj], (unsigned long long)__double_as_longlong(cn2[jj])};
    if (tid < 64) copy_of_lower[tid] = 0;
    bool copy = false;
    const int below = int(blockIdx.x) * 64 + 64;               // generators this workgroup has to look at
    for (int t0 = 0; t0 < below; t0 += TILE) {
        u64x2_t v[PER];
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int src = min(t0 + tid + 256 * q, k - 1);
            v[q] = u64x2_t{hash[src], (unsigned long long)__double_as_longlong(cn2[src])};
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PER; ++q) tile[tid + 256 * q] = v[q];
        __syncthreads();
        const int lim = min(TILE, j - t0);                     // only generators below j count
#pragma unroll 8
        for (int q = part; q < lim; q += 4) {
            const u64x2_t o = tile[q];
            copy |= (o.x == mine.x) & (o.y == mine.y);
        }
    }
    if (copy) copy_of_lower[tid & 63] = 1;
    __syncthreads();
    if (tid < 64 && j < k && copy_of_lower[tid]) rn[j] = 0.f;
}

// ------------------------------------------------------------------------------------------------
// Neighbourhood condition (Eq. 2): ||X_i - alpha_i C_f(i)||_2 <= eps ||X_i||_2, i.e. s(i,f(i)) >= (1 - eps^2) ||X_i||^2
// (the residual of a projection: ||X_i||^2 - s).  keep = 1 - eps^2; keep < 0 switches the test off (eps >= 1 can
// drop nothing).  In fp32 the test is trusted outside a band of 2^-11 ||X_i||^2 around the limit; inside it the
// token goes to the fp64 second look, which compares <X_i,C_j>^2 with keep ||X_i||^2 ||C_j||^2 (no division: a row
// that is an exact copy or power-of-two multiple of its generator passes at eps = 0 without rounding).
struct Neighbourhood {
    double keep;           // 1 - eps^2, or negative: no condition
    int* dropped;          // LDS counter of the workgroup

    // fp32 verdict on a token whose best score is s1 = m1^2: sure to be dropped / too close to call
    __device__ __forceinline__ void judge(float m1, float nx, bool& drop, bool& unsure) const {
        drop = unsure = false;
        if (keep >= 0.0) {
            const float s1 = m1 * m1, lim = float(keep) * nx, band = 0x1p-11f * nx;
            drop = s1 < lim - band;
            unsure = !drop && s1 < lim + band;
        }
    }
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

// The final word on one token, by one whole wave, in fp64: the best of its candidates by the score d^2 / ||C_j||^2
// (lowest j on a tie), then the neighbourhood condition, then f and alpha.  The candidates are every generator when
// `all` is set, else names[0..n) (a list in LDS, in any order), or the single generator j_single when names is null.
template <typename TR>
__device__ __noinline__ void second_look(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ C,
                                         const double* __restrict__ cn2, int nch, int k, int row, const int* names, int n, bool all,
                                         int j_single, Neighbourhood nb, int32_t* __restrict__ f, float* __restrict__ alpha) {
    const u32x4_t* xr = X + size_t(row) * nch;
    const int count = all ? k : (names ? n : 1);
    double bs = -1.0, bd = 0.0, bc = 1.0;
    int bj = 0;
    auto take = [&](int j, double d, double c2n) {
        const double sc = c2n > 0.0 ? d * d / c2n : 0.0;
        if (sc > bs || (sc == bs && j < bj)) { bs = sc; bd = d; bc = c2n; bj = j; }
    };
    auto cand = [&](int q) { return all ? q : (names ? names[q] : j_single); };
#pragma unroll 1
    for (int q = 0; q < count; q += 2) {
        const int ja = cand(q), jb = cand(min(q + 1, count - 1));
        const double na = cn2[ja], nbn = cn2[jb];            // in flight together with the rows
        double da, db;
        wave_dot2<TR>(xr, C + size_t(ja) * nch, C + size_t(jb) * nch, nch, da, db);
        take(ja, da, na);
        if (jb != ja) take(jb, db, nbn);
    }
    bool kept = true;
    if (nb.keep >= 0.0) {
        double nx, unused;
        wave_dot2<TR>(xr, xr, xr, nch, nx, unused);
        kept = bd * bd >= nb.keep * nx * bc;
    }
    if ((threadIdx.x & 63) == 0) {
        f[row] = bj;
        alpha[row] = (kept && bc > 0.0) ? float(bd / bc) : 0.f;
        if (!kept) atomicAdd(nb.dropped, 1);
    }
}

// ------------------------------------------------------------------------------------------------
// The scan of one token fragment on the accumulator registers.  D layout of the 32x32 MFMA: register i of lane (r,g)
// in generator fragment a is generator 32 a + 8 (i/4) + 4 g + (i%4) of the lane's generators, token r: the two lanes
// (r,0) and (r,1) hold the token's products with all of them.
__device__ __forceinline__ int lane_generator(int p, int g) { return 32 * (p >> 4) + 8 * ((p & 15) >> 2) + 4 * g + (p & 3); }

// r(i,j) = <X_i,C_j> / ||C_j|| replaces the products (sign kept; rn: the factors of this wave's generators in LDS);
// returns the largest and second largest |r| over the two lanes' generators, the lowest generator (numbered from
// jbase) attaining the largest, and the signed value there.  Both lanes of a token end up with the same values.
template <int NA, int NQ>
__device__ __forceinline__ void scan_fragment(f32x16_t (&acc)[NA][NQ], int tq, const float* rn, int g, int jbase, float& m1, float& m2,
                                              int& j1, float& a1) {
    m1 = -1.f; m2 = -1.f;
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 rn4 = *reinterpret_cast<const float4*>(&rn[32 * a + 8 * q + 4 * g]);
            const float rr[4] = {rn4.x, rn4.y, rn4.z, rn4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float v = acc[a][tq][4 * q + e] * rr[e];
                acc[a][tq][4 * q + e] = v;
                const float x = fabsf(v);
                m2 = __builtin_amdgcn_fmed3f(m1, x, m2);          // m2 <= m1 always: the median is the new second largest
                m1 = fmaxf(m1, x);
            }
        }
    // who attains the largest: walking down, the lowest position (= lowest generator of this lane) stays
    int p1 = 0;
    a1 = 0.f;
#pragma unroll
    for (int a = NA - 1; a >= 0; --a)
#pragma unroll
        for (int i = 15; i >= 0; --i) {
            const float v = acc[a][tq][i];
            const bool hit = fabsf(v) == m1;
            p1 = hit ? a * 16 + i : p1;
            a1 = hit ? v : a1;
        }
    j1 = jbase + lane_generator(p1, g);
    const float om1 = __shfl_xor(m1, 32), om2 = __shfl_xor(m2, 32), oa1 = __shfl_xor(a1, 32);
    const int oj1 = __shfl_xor(j1, 32);
    const bool other = om1 > m1 || (om1 == m1 && oj1 < j1);
    m2 = fmaxf(fminf(m1, om1), fmaxf(m2, om2));
    m1 = other ? om1 : m1;
    a1 = other ? oa1 : a1;
    j1 = other ? oj1 : j1;
}

// Names every generator of this lane whose |r| reaches lim (+infinity for lanes that have nothing to name) into the
// token's list in LDS: cnt[0] counts, names[0..kMaxNamed) takes the first ones.  One bit per register, then the set
// bits one by one: short straight-line code, because all of it misses the instruction cache.
template <int NA, int NQ>
__device__ __forceinline__ void name_fragment(const f32x16_t (&acc)[NA][NQ], int tq, float lim, int g, int jbase, int* cnt, int* names) {
#pragma unroll
    for (int a0 = 0; a0 < NA; a0 += 2) {
        uint32_t bits[2] = {0u, 0u};
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (a0 + h < NA) bits[h] |= (fabsf(acc[a0 + h][tq][i]) >= lim) ? (1u << i) : 0u;
        uint32_t todo = bits[0] | (bits[1] << 16);
        while (todo != 0u) {
            const int p = __ffs(int(todo)) - 1;              // fragment a0 + p / 16, register p % 16
            todo &= todo - 1u;
            const int slot = atomicAdd(cnt, 1);
            if (slot < kMaxNamed) names[slot] = jbase + lane_generator(16 * a0 + p, g);
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
// SKETCH: the same walk for the random-projection baseline (Sec. 4.6): the rows of C are the directions of the sketch,
// nothing is decided, and the epilogue stores the dot products themselves, S[i][j] = <X_i, C_j>, rounded once to the
// element type (rn, cn2, hash, cand, f, alpha, eta are not used).
template <typename TR, int TG, int TT, int NW, bool ALIGNED, bool FUSED, bool SKETCH = false>
__global__ __launch_bounds__(64 * NW) void k_score(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ C,
                                                   const float* __restrict__ rn, const double* __restrict__ cn2,
                                                   const unsigned long long* __restrict__ hash, int b, int nch, int k, int ncb,
                                                   u32x4_t* __restrict__ cand, int32_t* __restrict__ f, float* __restrict__ alpha,
                                                   double keep, int32_t* __restrict__ eta, void* __restrict__ sketch = nullptr) {
    static_assert(!(SKETCH && FUSED), "the sketch decides nothing");
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
    __shared__ __attribute__((aligned(16))) float lds_rn[GB];               // 1/||C_j||, 0 for generators that cannot win
    __shared__ unsigned long long lds_hash[FUSED ? GB : 1], lds_norm[FUSED ? GB : 1];
    __shared__ int drop_count;
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

    if (tid == 0) drop_count = 0;                              // published by the barriers of the main loop
    // The generators' factors 1/||C_j|| (0: cannot win); slots past the last generator count as generators that cannot
    // win.  With one column block the workgroup finds the copies among its generators itself (below, while its first
    // loads are in flight); with several, k_dedupe has done it.
    constexpr int GPT = (GB + NT - 1) / NT;       // generators per thread
    float rn_reg[GPT];
    unsigned long long hash_reg[GPT], norm_reg[GPT];
    if constexpr (!SKETCH) {
#pragma unroll
        for (int q = 0; q < GPT; ++q) {
            const int jj = min(gen0 + tid + NT * q, k - 1);
            rn_reg[q] = rn[jj];
            if (FUSED) { hash_reg[q] = hash[jj]; norm_reg[q] = (unsigned long long)__double_as_longlong(cn2[jj]); }
        }
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
    if constexpr (!SKETCH) {
#pragma unroll
        for (int q = 0; q < GPT; ++q) {
            const int t = tid + NT * q;
            if (t < GB) {
                lds_rn[t] = gen0 + t < k ? rn_reg[q] : 0.f;
                if (FUSED) { lds_hash[t] = hash_reg[q]; lds_norm[t] = norm_reg[q]; }
            }
        }
    }
    if (FUSED) {
        // a generator whose row is a bit-identical copy of a lower-numbered one (same hash, same fp64 norm) can never
        // win: lowest j takes a tie.  PARTS threads share the comparisons of one generator.
        __syncthreads();
        constexpr int PARTS = NT >= GB ? NT / GB : 1;
        for (int e = tid; e < GB * PARTS; e += NT) {
            const int t = e % GB, part = e / GB;
            const unsigned long long h = lds_hash[t], c2 = lds_norm[t];
            bool copy = false;
            for (int q = part; q < t; q += PARTS) copy |= (lds_hash[q] == h) & (lds_norm[q] == c2);
            if (copy) lds_rn[t] = 0.f;
        }
    }
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

    if constexpr (SKETCH) {
        // register i of fragment a belongs to direction gen0 + 32 a + 8 (i / 4) + 4 g + i % 4 and to token r of the
        // fragment: four consecutive directions of one token make one 8- or 16-byte store
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int row = row_base + 32 * tt + r;
#pragma unroll
            for (int a = 0; a < TG; ++a)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int j0 = gen0 + 32 * a + 8 * q + 4 * g;
                    if (row < b && j0 < k) {
                        const float v0 = acc[a][tt][4 * q], v1 = acc[a][tt][4 * q + 1], v2 = acc[a][tt][4 * q + 2],
                                    v3 = acc[a][tt][4 * q + 3];
                        if constexpr (TR::kElemBytes == 2) {
                            uint2 out;
                            out.x = pack_bf16(v0, v1);
                            out.y = pack_bf16(v2, v3);
                            *reinterpret_cast<uint2*>(static_cast<uint16_t*>(sketch) + size_t(row) * k + j0) = out;
                        } else {
                            *reinterpret_cast<float4*>(static_cast<float*>(sketch) + size_t(row) * k + j0) = make_float4(v0, v1, v2, v3);
                        }
                    }
                }
        }
        return;
    }

    // Epilogue: the scan runs on the accumulator registers themselves (scan_fragment).  Per wave a little LDS (all tiles
    // are free after the last barrier) takes the names of the generators that are too close to a token's best for fp32
    // to tell apart.
    int* const tok_cnt = reinterpret_cast<int*>(lds_raw) + wave * (32 * (1 + kMaxNamed));
    int* const tok_names = tok_cnt + 32;
    static_assert(NW * 32 * (1 + kMaxNamed) * sizeof(int) <= sizeof(lds_raw), "candidate lists do not fit");
    const Neighbourhood nb{keep, &drop_count};
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        float m1, m2, a1;
        int j1;
        scan_fragment(acc, tt, lds_rn, g, gen0, m1, m2, j1, a1);
        const int row = row_base + 32 * tt + r;
        const bool valid = row < b;
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
        // Too close to call in fp32: a second generator within the band.  Rare (about one token in a thousand), so the
        // wave only then walks its registers again, to name everybody within the band of each such token's best.
        const float thr = m1 * (1.f - kBand);
        const bool tie = valid && m1 > 0.f && m2 >= thr;
        int cnt = 0;
        if (__builtin_amdgcn_ballot_w64(tie) != 0ull) {
            if (lane < 32) tok_cnt[lane] = 0;
            wave_lds_sync();
            name_fragment(acc, tt, tie ? thr : __builtin_inff(), g, gen0, &tok_cnt[r], &tok_names[r * kMaxNamed]);
            wave_lds_sync();
            cnt = tie ? min(tok_cnt[r], kTooMany) : 0;
        }
        if (FUSED) {
            bool drop, close_call;
            nb.judge(m1, nx, drop, close_call);
            const bool unsure = valid && (tie || close_call);
            if (valid && !unsure && g == 0) {
                f[row] = j1;
                alpha[row] = drop ? 0.f : a1 * lds_rn[j1];              // one column block: gen0 = 0
                if (drop) atomicAdd(&drop_count, 1);
            }
            // the wave's undecided tokens, one after the other, in fp64 by the whole wave
            unsigned long long todo = __builtin_amdgcn_ballot_w64(unsure && g == 0);
            while (todo != 0ull) {
                const int t = __ffsll((long long)todo) - 1;             // lane = token number within the fragment
                todo &= todo - 1ull;
                const int row_t = __shfl(row, t), j_t = __shfl(j1, t), cnt_t = __shfl(cnt, t);
                second_look<TR>(X, C, cn2, nch, k, row_t, cnt_t > 0 ? tok_names + t * kMaxNamed : nullptr, cnt_t, cnt_t >= kTooMany,
                                j_t, nb, f, alpha);
            }
        } else if (valid && g == 0) {
            BlockRecord rec;
            rec.m1 = m1; rec.a1 = a1; rec.j1 = j1; rec.cnt = cnt;
#pragma unroll
            for (int q = 0; q < kMaxNamed; ++q) rec.names[q] = (q < cnt) ? tok_names[r * kMaxNamed + q] : 0;
            rec.store(cand + (size_t(row) * ncb + cb) * 2, nx);
        }
    }
    if (FUSED && want_norm) {
        __syncthreads();
        if (tid == 0 && drop_count > 0) atomicAdd(eta, drop_count);
    }
}

// ------------------------------------------------------------------------------------------------
// k_finalize: only needed when the generators span several column blocks.  One thread per token joins the blocks'
// records: the overall best, and every generator named within the band of it (a block's list holds all of its
// generators within the band of the BLOCK's best, which reaches at least as far down).  A token with a single
// candidate is decided on the spot; the others wait in LDS for the workgroup's waves, which re-decide them in fp64.
constexpr int kMaxMerged = 8;                   // candidates of one token over all blocks; more: every generator again
constexpr int kEntryInts = 3 + kMaxMerged;      // row, number of names (0: only the neighbourhood condition is in doubt; -1: all), j1, names

template <typename TR>
__global__ __launch_bounds__(256) void k_finalize(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ C,
                                                  const float* __restrict__ rn, const double* __restrict__ cn2,
                                                  const u32x4_t* __restrict__ cand, int b, int nch, int k, int ncb,
                                                  int32_t* __restrict__ f, float* __restrict__ alpha, double keep,
                                                  int32_t* __restrict__ eta) {
    __shared__ int q_count, drop_count;
    __shared__ int q_list[256];
    __shared__ int entries[256 * kEntryInts];           // one slot per thread; q_list names the slots in use
    const int tid = threadIdx.x, row = blockIdx.x * 256 + tid;
    if (tid == 0) { q_count = 0; drop_count = 0; }
    __syncthreads();
    const Neighbourhood nb{keep, &drop_count};
    if (row < b) {
        const u32x4_t* recs = cand + size_t(row) * ncb * 2;
        float m1 = -1.f, a1 = 0.f;
        int j1 = 0;
        for (int cb = 0; cb < ncb; ++cb) {
            BlockRecord rec;
            rec.load_lead(recs + 2 * cb);
            if (rec.m1 > m1 || (rec.m1 == m1 && rec.j1 < j1)) { m1 = rec.m1; a1 = rec.a1; j1 = rec.j1; }
        }
        int* e = entries + tid * kEntryInts;
        int n = 0;
        bool many = false;
        auto add = [&](int j) {
            if (n < kMaxMerged) e[3 + n++] = j; else many = true;
        };
        if (m1 > 0.f) {
            const float thr = m1 * (1.f - kBand);
            for (int cb = 0; cb < ncb; ++cb) {
                BlockRecord rec;
                rec.load_lead(recs + 2 * cb);
                if (rec.m1 < thr) continue;
                if (rec.cnt == 0) { add(rec.j1); continue; }
                if (rec.cnt > kMaxNamed) { many = true; continue; }
                rec.load_rest(recs + 2 * cb);
#pragma unroll
                for (int q = 0; q < kMaxNamed; ++q)
                    if (q < rec.cnt) add(rec.names[q]);
            }
        }
        const bool tie = many || n > 1;
        const float nx = keep >= 0.0 ? BlockRecord::load_norm(recs) : 0.f;      // every block stores the same value
        bool drop, close_call;
        nb.judge(m1, nx, drop, close_call);
        if (!tie && !close_call) {
            f[row] = j1;
            alpha[row] = drop ? 0.f : a1 * rn[j1];
            if (drop) atomicAdd(&drop_count, 1);
        } else {
            e[0] = row; e[1] = tie ? (many ? -1 : n) : 0; e[2] = j1;
            q_list[atomicAdd(&q_count, 1)] = tid;
        }
    }
    __syncthreads();
    const int total = q_count;
    for (int t = tid >> 6; t < total; t += 4) {
        const int* e = entries + q_list[t] * kEntryInts;
        const int n = e[1];
        second_look<TR>(X, C, cn2, nch, k, e[0], n != 0 ? e + 3 : nullptr, n, n < 0, e[2], nb, f, alpha);
    }
    if (keep >= 0.0) {
        __syncthreads();
        if (tid == 0 && drop_count > 0) atomicAdd(eta, drop_count);
    }
}

// ------------------------------------------------------------------------------------------------ host side

struct ScoreArgs {
    const void* X; const void* C; const float* rn; const double* cn2; const unsigned long long* hash;
    int b, nch, k;
    u32x4_t* cand; int32_t* f; float* alpha;
    double keep; int32_t* eta;
};

template <typename TR, int TG, int TT, int NW, bool FUSED>
static void launch_score_cfg(const CompressPlan& pl, const ScoreArgs& a, hipStream_t s) {
    dim3 grid((unsigned)(pl.ncb > 1 ? (pl.row_tiles + 7) / 8 * 8 * pl.ncb : pl.row_tiles));
    if (a.nch % 8 == 0)      // every row is a whole number of 128-byte super-steps
        hipLaunchKernelGGL((k_score<TR, TG, TT, NW, true, FUSED>), grid, dim3(64 * NW), 0, s, (const u32x4_t*)a.X,
                           (const u32x4_t*)a.C, a.rn, a.cn2, a.hash, a.b, a.nch, a.k, pl.ncb, a.cand, a.f, a.alpha, a.keep, a.eta);
    else
        hipLaunchKernelGGL((k_score<TR, TG, TT, NW, false, FUSED>), grid, dim3(64 * NW), 0, s, (const u32x4_t*)a.X,
                           (const u32x4_t*)a.C, a.rn, a.cn2, a.hash, a.b, a.nch, a.k, pl.ncb, a.cand, a.f, a.alpha, a.keep, a.eta);
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

// The sketch S = X Pt^T on the walk of the score kernel; the plan is the one the score kernel would take for r generators.
template <typename TR, int TG, int NW>
static void launch_sketch_cfg(const CompressPlan& pl, const void* X, const void* Pt, int b, int nch, int r, void* S, hipStream_t s) {
    dim3 grid((unsigned)(pl.ncb > 1 ? (pl.row_tiles + 7) / 8 * 8 * pl.ncb : pl.row_tiles));
#define PAMM_LAUNCH_SKETCH(AL) \
    hipLaunchKernelGGL((k_score<TR, TG, 1, NW, AL, false, true>), grid, dim3(64 * NW), 0, s, (const u32x4_t*)X, (const u32x4_t*)Pt, \
                       (const float*)nullptr, (const double*)nullptr, (const unsigned long long*)nullptr, b, nch, r, pl.ncb,        \
                       (u32x4_t*)nullptr, (int32_t*)nullptr, (float*)nullptr, -1.0, (int32_t*)nullptr, S)
    if (nch % 8 == 0) PAMM_LAUNCH_SKETCH(true);
    else PAMM_LAUNCH_SKETCH(false);
#undef PAMM_LAUNCH_SKETCH
}

template <typename TR>
static void launch_sketch(const CompressPlan& pl, const void* X, const void* Pt, int b, int nch, int r, void* S, hipStream_t s) {
    // r <= 128: at most four fragments per wave; the waves per workgroup are the plan's
#define PAMM_SKETCH_NW(TGV)                                                             \
    do {                                                                                \
        if (pl.nw == 8) launch_sketch_cfg<TR, TGV, 8>(pl, X, Pt, b, nch, r, S, s);      \
        else if (pl.nw == 4) launch_sketch_cfg<TR, TGV, 4>(pl, X, Pt, b, nch, r, S, s); \
        else launch_sketch_cfg<TR, TGV, 2>(pl, X, Pt, b, nch, r, S, s);                 \
    } while (0)
    if (pl.tg == 1) PAMM_SKETCH_NW(1);
    else if (pl.tg == 2) PAMM_SKETCH_NW(2);
    else PAMM_SKETCH_NW(4);
#undef PAMM_SKETCH_NW
}

// idx_dev: the generators' row numbers in device memory, or NULL: then idx_host holds them (host memory, only read
// during the call) and they travel in argument blocks.
template <typename TR>
static pamm_status run_compress(const CompressPlan& pl, const void* X, int b, int n, int k, const int32_t* idx_dev,
                                const int32_t* idx_host, double keep, void* C, int32_t* f, float* alpha, int32_t* eta, char* ws,
                                hipStream_t s) {
    const int nch = n / TR::kPerChunk;
    int32_t* idx = reinterpret_cast<int32_t*>(ws + pl.off_idx);
    float* rn = reinterpret_cast<float*>(ws + pl.off_rn);
    double* cn2 = reinterpret_cast<double*>(ws + pl.off_cn2);
    unsigned long long* hash = reinterpret_cast<unsigned long long*>(ws + pl.off_hash);
    u32x4_t* cand = reinterpret_cast<u32x4_t*>(ws + pl.off_cand);

    {
        ScopedSpan span(kGather, s);
        if (idx_dev) {
            hipLaunchKernelGGL((k_gather<TR>), dim3(k), dim3(256), 0, s, (const u32x4_t*)X, idx_dev, b, nch, (u32x4_t*)C, idx, rn, cn2,
                               hash, eta);
        } else {
            for (int j0 = 0; j0 < k; j0 += kArgGenerators) {
                const int cnt = k - j0 < kArgGenerators ? k - j0 : kArgGenerators;
                IdxByValue ia;
                for (int j = 0; j < kArgGenerators; ++j) ia.v[j] = j < cnt ? idx_host[j0 + j] : 0;
                hipLaunchKernelGGL((k_gather_arg<TR>), dim3(cnt), dim3(256), 0, s, (const u32x4_t*)X, ia, j0, b, nch, (u32x4_t*)C, idx,
                                   rn, cn2, hash, eta);
            }
        }
        if (pl.ncb > 1)
            hipLaunchKernelGGL(k_dedupe, dim3((k + 63) / 64), dim3(256), 0, s, cn2, hash, k, rn);
    }
    {
        ScopedSpan span(kScore, s);
        launch_score<TR>(pl, ScoreArgs{X, C, rn, cn2, hash, b, nch, k, cand, f, alpha, keep, eta}, s);
    }
    if (pl.ncb > 1) {
        ScopedSpan span(kFinalize, s);
        hipLaunchKernelGGL((k_finalize<TR>), dim3((b + 255) / 256), dim3(256), 0, s, (const u32x4_t*)X, (const u32x4_t*)C, rn, cn2,
                           cand, b, nch, k, pl.ncb, f, alpha, keep, eta);
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

extern "C" pamm_status pamm_sketch(const void* X, const void* Pt, int64_t b, int64_t n, int64_t r, pamm_dtype dt, void* S,
                                   void* stream) {
    pamm_status st = check_sketch_args(X, Pt, b, n, r, dt, S);
    if (st != PAMM_OK) return st;
    CompressPlan pl;
    st = plan_compress(b, n, r, dt, &pl);
    if (st != PAMM_OK) return st;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    ScopedSpan span(kSketch, s);
    if (dt == PAMM_BF16) launch_sketch<Bf16>(pl, X, Pt, int(b), int(n / 8), int(r), S, s);
    else launch_sketch<F32>(pl, X, Pt, int(b), int(n / 4), int(r), S, s);
    return hipGetLastError() == hipSuccess ? PAMM_OK : PAMM_ERR_DEVICE;
}
