// pamm_compress / pamm_compress_idx: Alg. 1, procedure Compress, at eps = infinity.
//
// Three launches on the caller's stream:
//   k_gather    C_j = X[idx_j] (bit copy), ||C_j||^2 in fp64, a content hash per generator
//   k_score     streams X once; D = C X^T on the matrix cores with C staged through LDS, then per token the
//               three largest distinct values of s(i,j) = <X_i,C_j>^2/||C_j||^2 (Lemma 1) and where they occur
//   k_finalize  merges column blocks, writes f and alpha (Eq. 1), and re-decides in fp64 the few rows whose
//               leading scores are too close for fp32 to separate
#include <hip/hip_runtime.h>

#include <mutex>
#include <vector>

#include "pamm_device.h"
#include "pamm_plan.h"
#include "pamm_profile.h"

namespace pamm {

// ------------------------------------------------------------------------------------------------
// Per-token running record of the best generators seen so far.  Equal scores are not listed twice:
// s1 > s2 > s3 are the three largest DISTINCT score values; j1 / j2 are the lowest generator numbers
// attaining s1 / s2; jt is the lowest generator other than j1 that attains s1 exactly (-1 if none).
// Bit-identical generators (padding tokens sampled twice) produce bit-identical scores, so they meet
// in jt instead of hiding the real runner-up.
struct Best {
    float s1; int j1; float d1; int jt; float s2; int j2; float s3;

    __device__ __forceinline__ void init() { s1 = -1.f; j1 = 0; d1 = 0.f; jt = -1; s2 = -2.f; j2 = 0; s3 = -3.f; }

    // generators arrive in increasing j
    __device__ __forceinline__ void push(float s, int j, float d) {
        if (s > s1) { s3 = s2; s2 = s1; j2 = j1; s1 = s; j1 = j; d1 = d; jt = -1; }
        else if (s == s1) { if (jt < 0) jt = j; }
        else if (s > s2) { s3 = s2; s2 = s; j2 = j; }
        else if (s < s2 && s > s3) { s3 = s; }
    }

    __device__ __forceinline__ void insert_lower(float s, int j) {   // s < s1
        if (s > s2) { s3 = s2; s2 = s; j2 = j; }
        else if (s == s2) { j2 = min(j2, j); }
        else if (s > s3) { s3 = s; }
    }

    // union with a record built over a disjoint set of generators
    __device__ __forceinline__ void merge(const Best& o) {
        if (o.s1 > s1) {
            s3 = s2; s2 = s1; j2 = j1;
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
        if (o.s3 < s2 && o.s3 > s3) s3 = o.s3;
    }
};

// ------------------------------------------------------------------------------------------------
// k_gather: one workgroup per generator.
template <typename TR>
__global__ __launch_bounds__(256) void k_gather(const u32x4_t* __restrict__ X, const int32_t* __restrict__ idx_in, int b, int nch,
                                                u32x4_t* __restrict__ C, int32_t* __restrict__ idx_out, float* __restrict__ inv,
                                                double* __restrict__ cn2, unsigned long long* __restrict__ hash) {
    const int j = blockIdx.x;
    int src = idx_in[j];
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

// ------------------------------------------------------------------------------------------------
// k_score.  Workgroup = 4 waves; wave w owns 32*TT tokens; the workgroup owns one column block of
// 32*TG generators.  Roles in the 32x32 MFMA: A operand = generators, B operand = tokens, so a lane
// ends up holding scores of ONE token (lane%32) against 16*TG generators per token fragment and the
// argmax runs in registers; only the two half-waves have to be merged at the end.
//
// The hidden dimension is walked in "super-steps" of 8 chunks (128 bytes of a row): lane (r,g) loads
// the 64 contiguous bytes [64g, 64g+64) of that window from its row, i.e. 4 chunks that feed 4
// MFMA K-steps.  Which hidden index lands in which K slot is irrelevant for a dot product as long
// as the generator operand uses the same map, which it does (same (g,u) -> chunk rule).
//
// C is staged through LDS in stages of 64/TG chunks per generator (32 KiB per stage), double
// buffered: global loads of stage s+1 are in flight while stage s is consumed.
template <typename TR, int TG, int TT, bool ALIGNED>
__global__ __launch_bounds__(256) void k_score(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ C,
                                               const float* __restrict__ inv, int b, int nch, int k, int ncb,
                                               u32x4_t* __restrict__ cand) {
    constexpr int GB = 32 * TG;          // generators per column block
    constexpr int SS = 8 / TG;           // super-steps per stage
    constexpr int CPS = 8 * SS;          // chunks per generator per stage
    constexpr int RS = CPS + 1;          // LDS row stride in chunks (odd: conflict-free 16-byte reads down a column)
    constexpr int LOADS = GB * CPS / 256;   // = 8 chunks per thread per stage

    __shared__ u32x4_t lds_c[2][GB * RS];
    __shared__ float lds_inv[GB];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, r = lane & 31, g = lane >> 5;
    const int cb = blockIdx.x % ncb;
    const int rt = blockIdx.x / ncb;
    const int gen0 = cb * GB;

    if (tid < GB) {
        int j = gen0 + tid;
        lds_inv[tid] = j < k ? inv[j] : -1.f;      // negative marks a slot past the last generator
    }

    // token rows of this lane (clamped: rows past the end are computed on a valid row and never stored)
    const int row_base = rt * (128 * TT) + wave * (32 * TT);
    const u32x4_t* xrow[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        int row = row_base + 32 * tt + r;
        row = row < b ? row : b - 1;
        xrow[tt] = X + size_t(row) * nch;
    }

    f32x16_t acc[TG][TT];
#pragma unroll
    for (int a = 0; a < TG; ++a)
#pragma unroll
        for (int t = 0; t < TT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][t][i] = 0.f;

    const int nstages = (nch + CPS - 1) / CPS;
    const int nss = (nch + 7) / 8;               // super-steps

    u32x4_t creg[LOADS];
    auto load_c = [&](int stage) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            int q = tid + 256 * i;
            int row = q / CPS, cc = q % CPS;
            const int j = gen0 + row, c = stage * CPS + cc;
            // Clamped addresses, no guard and no mask: a guarded load costs a branch per chunk, and a mask makes
            // the compiler wait for the load where it is issued.  Rows past the last generator are ignored by
            // the epilogue; chunks past the end of a row meet zero chunks of X.
            creg[i] = C[size_t(min(j, k - 1)) * nch + min(c, nch - 1)];
        }
    };
    auto store_c = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            int q = tid + 256 * i;
            lds_c[buf][(q / CPS) * RS + (q % CPS)] = creg[i];
        }
    };
    // X ring: D super-steps of this lane's chunks live in registers; loads run D-1 super-steps ahead of the
    // MFMAs so that every wave keeps (D-1) * TT * 4 KiB of X in flight.
    constexpr int D = (TG * TT >= 16) ? 2 : 4;
    constexpr int UN = SS > D ? SS : D;          // super-steps per unrolled body: a multiple of SS and of D
    u32x4_t xr[D][TT][4];
    auto load_x = [&](u32x4_t (&dst)[TT][4], int sstep) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (ALIGNED) {        // rows are whole super-steps: clamp the super-step, nothing to mask
#if defined(PAMM_DBG_NOX)
                    dst[tt][u] = u32x4_t{uint32_t(sstep), 1u, 2u, 3u};
#else
                    dst[tt][u] = xrow[tt][min(sstep, nss - 1) * 8 + 4 * g + u];
#endif
                } else {
                    const int c = sstep * 8 + 4 * g + u;
                    const uint32_t keep = c < nch ? 0xffffffffu : 0u;
                    dst[tt][u] = xrow[tt][min(c, nch - 1)] & keep;
                }
            }
    };

    load_c(0);
#pragma unroll
    for (int d = 0; d < D - 1; ++d) load_x(xr[d], d);
    store_c(0);
    __syncthreads();

    const int nbody = (nss + UN - 1) / UN;
    int buf = 0, stage = 0;
    for (int bi = 0; bi < nbody; ++bi) {
#pragma unroll
        for (int p = 0; p < UN; ++p) {
            const int gs = bi * UN + p;                      // super-step
            if (p % SS == 0) {                               // a stage of C begins
                stage = gs / SS;
                if (stage + 1 < nstages) load_c(stage + 1);
            }
            load_x(xr[(p + D - 1) % D], gs + D - 1);
            if (gs < nss) {                                  // uniform; only false in the tail of the last body
                const u32x4_t* cbuf = lds_c[buf];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    u32x4_t a[TG];
#pragma unroll
                    for (int tg = 0; tg < TG; ++tg) a[tg] = cbuf[(32 * tg + r) * RS + (p % SS) * 8 + 4 * g + u];
#pragma unroll
                    for (int tg = 0; tg < TG; ++tg)
#pragma unroll
                        for (int tt = 0; tt < TT; ++tt) {
#if defined(PAMM_DBG_NOMMA)
                            acc[tg][tt][0] += __uint_as_float(a[tg].x ^ xr[p % D][tt][u].x);
#else
                            TR::mma(a[tg], xr[p % D][tt][u], acc[tg][tt]);
#endif
                        }
                }
            }
            if (p % SS == SS - 1) {                          // the stage ends: publish the next one
                if (stage + 1 < nstages) store_c(buf ^ 1);
                __syncthreads();
                buf ^= 1;
            }
        }
    }

    // epilogue: D layout of the 32x32 MFMA: register i of lane (r,g) is generator 8*(i/4)+4*g+(i%4), token r
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        Best best;
        best.init();
#pragma unroll
        for (int tg = 0; tg < TG; ++tg) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                int jl = 32 * tg + 8 * (i >> 2) + 4 * g + (i & 3);
                float iv = lds_inv[jl];
                float d = acc[tg][tt][i];
                float s = d * d * iv;
                if (iv >= 0.f) best.push(s, gen0 + jl, d);
            }
        }
        Best o;
        o.s1 = __shfl_xor(best.s1, 32); o.j1 = __shfl_xor(best.j1, 32); o.d1 = __shfl_xor(best.d1, 32);
        o.jt = __shfl_xor(best.jt, 32); o.s2 = __shfl_xor(best.s2, 32); o.j2 = __shfl_xor(best.j2, 32);
        o.s3 = __shfl_xor(best.s3, 32);
        best.merge(o);
        int row = row_base + 32 * tt + r;
        if (g == 0 && row < b) {
            u32x4_t* dst = cand + (size_t(row) * ncb + cb) * 2;
            dst[0] = u32x4_t{__float_as_uint(best.s1), uint32_t(best.j1), __float_as_uint(best.d1), uint32_t(best.jt)};
            dst[1] = u32x4_t{__float_as_uint(best.s2), uint32_t(best.j2), __float_as_uint(best.s3), 0u};
        }
    }
}

// ------------------------------------------------------------------------------------------------
// k_finalize: one thread per token.
template <typename TR>
__device__ __forceinline__ double wave_dot(const u32x4_t* __restrict__ x, const u32x4_t* __restrict__ c, int nch, int lane) {
    double acc = 0.0;
    for (int q = lane; q < nch; q += kWave) {
        float a[TR::kPerChunk], bq[TR::kPerChunk];
        TR::unpack(x[q], a);
        TR::unpack(c[q], bq);
#pragma unroll
        for (int e = 0; e < TR::kPerChunk; ++e) acc += double(a[e]) * double(bq[e]);
    }
    return wave_sum(acc);
}

template <typename TR>
__global__ __launch_bounds__(256) void k_finalize(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ C,
                                                  const float* __restrict__ inv, const double* __restrict__ cn2,
                                                  const unsigned long long* __restrict__ hash,
                                                  const u32x4_t* __restrict__ cand, int b, int nch, int k, int ncb,
                                                  int32_t* __restrict__ f, float* __restrict__ alpha) {
    const int row = blockIdx.x * 256 + threadIdx.x;
    const int lane = threadIdx.x & 63;
    const bool valid = row < b;
    Best st;
    st.init();
    if (valid) {
        for (int cb = 0; cb < ncb; ++cb) {
            const u32x4_t* src = cand + (size_t(row) * ncb + cb) * 2;
            u32x4_t p = src[0], q = src[1];
            Best o;
            o.s1 = __uint_as_float(p.x); o.j1 = int(p.y); o.d1 = __uint_as_float(p.z); o.jt = int(p.w);
            o.s2 = __uint_as_float(q.x); o.j2 = int(q.y); o.s3 = __uint_as_float(q.z);
            if (cb == 0) st = o; else st.merge(o);
        }
    }
    int fi = st.j1;
    float al = st.d1 * inv[st.j1];
    // 0: fp32 decision stands; 1: re-decide between two generators in fp64; 2: re-decide among all generators
    int mode = 0, other = st.j2;
    if (valid && st.s1 > 0.f) {
        const float thr = st.s1 * (1.f - 0x1p-12f);
        bool tie_other = false;
        if (st.jt >= 0)
            tie_other = !(hash[st.j1] == hash[st.jt] && __double_as_longlong(cn2[st.j1]) == __double_as_longlong(cn2[st.jt]));
        const bool close2 = st.s2 >= thr, close3 = st.s3 >= thr;
        if (tie_other || close2) {
            mode = (close3 || (tie_other && close2)) ? 2 : 1;
            other = tie_other ? st.jt : st.j2;
        }
    }
    unsigned long long pending = __ballot(mode != 0);
    while (pending) {
        const int L = __ffsll((long long)pending) - 1;
        pending &= pending - 1;
        const int rrow = __shfl(row, L), rmode = __shfl(mode, L);
        const int ja = __shfl(st.j1, L), jb = __shfl(other, L);
        const u32x4_t* xr = X + size_t(rrow) * nch;
        double bs = -1.0, bd = 0.0, bc = 1.0;
        int bj = 0;
        auto eval = [&](int j) {
            double d = wave_dot<TR>(xr, C + size_t(j) * nch, nch, lane);
            double c2 = cn2[j];
            double s = c2 > 0.0 ? d * d / c2 : 0.0;
            if (s > bs) { bs = s; bd = d; bc = c2; bj = j; }       // strict: lowest j keeps a tie
        };
        if (rmode == 1) {
            eval(min(ja, jb));
            eval(max(ja, jb));
        } else {
            for (int j = 0; j < k; ++j) eval(j);
        }
        if (lane == L) {
            fi = bj;
            al = bc > 0.0 ? float(bd / bc) : 0.f;
        }
    }
    if (valid) {
        f[row] = fi;
        alpha[row] = al;
    }
}

// ------------------------------------------------------------------------------------------------ host side

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <typename TR, int TG>
static void launch_score_tt(const CompressPlan& pl, const void* X, const void* C, const float* inv, int b, int nch, int k,
                            u32x4_t* cand, hipStream_t s) {
    dim3 grid((unsigned)(pl.row_tiles * pl.ncb));
    const bool aligned = nch % 8 == 0;      // every row is a whole number of 128-byte super-steps
#define PAMM_LAUNCH_SCORE(TTV, AL) \
    hipLaunchKernelGGL((k_score<TR, TG, TTV, AL>), grid, dim3(256), 0, s, (const u32x4_t*)X, (const u32x4_t*)C, inv, b, nch, k, pl.ncb, cand)
    if (pl.tt == 2) { if (aligned) PAMM_LAUNCH_SCORE(2, true); else PAMM_LAUNCH_SCORE(2, false); }
    else            { if (aligned) PAMM_LAUNCH_SCORE(1, true); else PAMM_LAUNCH_SCORE(1, false); }
#undef PAMM_LAUNCH_SCORE
}

template <typename TR>
static void launch_score(const CompressPlan& pl, const void* X, const void* C, const float* inv, int b, int nch, int k,
                         u32x4_t* cand, hipStream_t s) {
    switch (pl.tg) {
        case 1: launch_score_tt<TR, 1>(pl, X, C, inv, b, nch, k, cand, s); break;
        case 2: launch_score_tt<TR, 2>(pl, X, C, inv, b, nch, k, cand, s); break;
        case 4: launch_score_tt<TR, 4>(pl, X, C, inv, b, nch, k, cand, s); break;
        default: launch_score_tt<TR, 8>(pl, X, C, inv, b, nch, k, cand, s); break;
    }
}

template <typename TR>
static pamm_status run_compress(const CompressPlan& pl, const void* X, int b, int n, int k, const int32_t* idx_src,
                                void* C, int32_t* f, float* alpha, char* ws, hipStream_t s) {
    const int nch = n / TR::kPerChunk;
    int32_t* idx = reinterpret_cast<int32_t*>(ws + pl.off_idx);
    float* inv = reinterpret_cast<float*>(ws + pl.off_inv);
    double* cn2 = reinterpret_cast<double*>(ws + pl.off_cn2);
    unsigned long long* hash = reinterpret_cast<unsigned long long*>(ws + pl.off_hash);
    u32x4_t* cand = reinterpret_cast<u32x4_t*>(ws + pl.off_cand);

    {
        ScopedSpan span(kGather, s);
        hipLaunchKernelGGL((k_gather<TR>), dim3(k), dim3(256), 0, s, (const u32x4_t*)X, idx_src, b, nch, (u32x4_t*)C, idx, inv, cn2, hash);
    }
    {
        ScopedSpan span(kScore, s);
        launch_score<TR>(pl, X, C, inv, b, nch, k, cand, s);
    }
    {
        ScopedSpan span(kFinalize, s);
        hipLaunchKernelGGL((k_finalize<TR>), dim3((b + 255) / 256), dim3(256), 0, s, (const u32x4_t*)X, (const u32x4_t*)C, inv, cn2,
                           hash, cand, b, nch, k, pl.ncb, f, alpha);
    }
    return hipGetLastError() == hipSuccess ? PAMM_OK : PAMM_ERR_DEVICE;
}

static pamm_status check_compress_args(const void* X, int64_t b, int64_t n, int64_t k, pamm_dtype dt, void* C, int32_t* f,
                                       float* alpha, void* ws, size_t ws_bytes, CompressPlan* pl) {
    pamm_status st = plan_compress(b, n, k, dt, pl);
    if (st != PAMM_OK) return st;
    if (!X || !C || !f || !alpha) return PAMM_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(C) || !aligned16(f) || !aligned16(alpha)) return PAMM_ERR_INVALID_ARG;
    if (!ws || ws_bytes < pl->total) return PAMM_ERR_WORKSPACE;
    if (!aligned16(ws)) return PAMM_ERR_INVALID_ARG;
    return PAMM_OK;
}

// ---- pinned ring that carries sampled indices to the gather kernel without a copy or a sync ----
constexpr int kRingSlots = 32;
constexpr int kMaxDevices = 16;
struct IdxRing {
    int32_t* host = nullptr;
    int32_t* dev = nullptr;
    hipEvent_t ev[kRingSlots];
    bool used[kRingSlots] = {};
    int next = 0;
    bool ready = false;
};
static IdxRing g_ring[kMaxDevices];
static std::mutex g_ring_mu;

}  // namespace pamm

using namespace pamm;

extern "C" pamm_status pamm_compress_idx(const void* X, int64_t b, int64_t n, int64_t k, const int32_t* idx_dev, pamm_dtype dt,
                                         void* C, int32_t* f, float* alpha, void* ws, size_t ws_bytes, void* stream) {
    CompressPlan pl;
    pamm_status st = check_compress_args(X, b, n, k, dt, C, f, alpha, ws, ws_bytes, &pl);
    if (st != PAMM_OK) return st;
    if (!idx_dev) return PAMM_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (dt == PAMM_BF16) return run_compress<Bf16>(pl, X, int(b), int(n), int(k), idx_dev, C, f, alpha, (char*)ws, s);
    return run_compress<F32>(pl, X, int(b), int(n), int(k), idx_dev, C, f, alpha, (char*)ws, s);
}

extern "C" pamm_status pamm_compress(const void* X, int64_t b, int64_t n, int64_t k, uint64_t seed, pamm_dtype dt, void* C,
                                     int32_t* f, float* alpha, void* ws, size_t ws_bytes, void* stream) {
    CompressPlan pl;
    pamm_status st = check_compress_args(X, b, n, k, dt, C, f, alpha, ws, ws_bytes, &pl);
    if (st != PAMM_OK) return st;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);

    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return PAMM_ERR_DEVICE;

    std::lock_guard<std::mutex> lock(g_ring_mu);
    IdxRing& ring = g_ring[device];
    if (!ring.ready) {
        void* h = nullptr;
        if (hipHostMalloc(&h, size_t(kRingSlots) * kMaxGenerators * sizeof(int32_t), hipHostMallocDefault) != hipSuccess)
            return PAMM_ERR_DEVICE;
        void* d = nullptr;
        if (hipHostGetDevicePointer(&d, h, 0) != hipSuccess) { (void)hipHostFree(h); return PAMM_ERR_DEVICE; }
        for (int i = 0; i < kRingSlots; ++i)
            if (hipEventCreateWithFlags(&ring.ev[i], hipEventDisableTiming) != hipSuccess) return PAMM_ERR_DEVICE;
        ring.host = static_cast<int32_t*>(h);
        ring.dev = static_cast<int32_t*>(d);
        ring.ready = true;
    }
    const int slot = ring.next;
    ring.next = (ring.next + 1) % kRingSlots;
    // a slot is reused only after the gather kernel that read it has finished (32 calls ago: normally long done)
    if (ring.used[slot] && hipEventSynchronize(ring.ev[slot]) != hipSuccess) return PAMM_ERR_DEVICE;
    int32_t* hidx = ring.host + size_t(slot) * kMaxGenerators;
    st = pamm_sample_indices(b, k, seed, hidx);
    if (st != PAMM_OK) return st;
    const int32_t* didx = ring.dev + size_t(slot) * kMaxGenerators;

    if (dt == PAMM_BF16) st = run_compress<Bf16>(pl, X, int(b), int(n), int(k), didx, C, f, alpha, (char*)ws, s);
    else st = run_compress<F32>(pl, X, int(b), int(n), int(k), didx, C, f, alpha, (char*)ws, s);
    if (hipEventRecord(ring.ev[slot], s) != hipSuccess) return PAMM_ERR_DEVICE;
    ring.used[slot] = true;
    return st;
}
