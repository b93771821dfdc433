// pamm_grad / pamm_contract: Alg. 1, procedure ApproxMM.
//
// Three launches on the caller's stream:
//   k_group     stable grouping of the rows by f(i): workgroup j lists the rows of generator j in increasing i
//               and cuts the list into pieces of at most P rows
//   k_contract  streams dY once: one wave per (piece, 512 columns) sums alpha_i * dY_i in registers, in list
//               order, and writes one fp32 partial row.  No atomics, no LDS; bit-reproducible.
//   k_ctb       dW = C^T Btilde on the matrix cores; Btilde_j is formed on the fly as the sum of generator j's
//               partial rows
#include <hip/hip_runtime.h>

#include "pamm_device.h"
#include "pamm_plan.h"
#include "pamm_profile.h"

namespace pamm {

// ------------------------------------------------------------------------------------------------
// k_group.  grid = k, 1024 threads.  Every workgroup reads all of f twice (f is b int32: it stays in
// L2): pass 1 counts rows with key < j (start of generator j's list) and key == j per wave, pass 2
// compacts the matching row numbers with ballots, which keeps them in increasing order.
// Slot table: generator j owns slots [seg_start_j / P + j, ... + ceil(count_j / P)); these ranges are
// disjoint and fit in floor(b/P) + k slots; slots between two generators' ranges are marked empty here.
__device__ __forceinline__ void load_keys(const int32_t* __restrict__ f, int i0, int b, int k, int (&key)[4]) {
    if (i0 + 3 < b) {
        int4 v = *reinterpret_cast<const int4*>(f + i0);
        key[0] = v.x; key[1] = v.y; key[2] = v.z; key[3] = v.w;
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) key[c] = (i0 + c < b) ? f[i0 + c] : -1;
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        bool in = i0 + c < b;
        int v = key[c];
        v = v < 0 ? 0 : (v >= k ? k - 1 : v);
        key[c] = in ? v : k;            // k = "no row": larger than every generator number
    }
}

__global__ __launch_bounds__(1024) void k_group(const int32_t* __restrict__ f, const float* __restrict__ alpha, int b, int k,
                                                int P, int nslots, int32_t* __restrict__ perm, float* __restrict__ alpha_s,
                                                int32_t* __restrict__ slot_row0, int32_t* __restrict__ slot_len,
                                                int32_t* __restrict__ sbase, int32_t* __restrict__ snum) {
    const int j = blockIdx.x;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const long long per_wave = (((long long)b + 15) / 16 + 255) / 256 * 256;
    const long long r0l = per_wave * wave;
    const int r0 = r0l < b ? int(r0l) : b;
    const int r1 = (r0l + per_wave) < b ? int(r0l + per_wave) : b;

    int lt = 0, eq = 0;
    for (int base = r0; base < r1; base += 256) {
        int key[4];
        load_keys(f, base + 4 * lane, b, k, key);
#pragma unroll
        for (int c = 0; c < 4; ++c) { lt += key[c] < j; eq += key[c] == j; }
    }
    lt = wave_sum(lt);
    eq = wave_sum(eq);
    __shared__ int s_lt[16], s_eq[16];
    if (lane == 0) { s_lt[wave] = lt; s_eq[wave] = eq; }
    __syncthreads();
    int seg_start = 0, count = 0, woff = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        seg_start += s_lt[w];
        woff += (w < wave) ? s_eq[w] : 0;
        count += s_eq[w];
    }

    int pos = seg_start + woff;
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int base = r0; base < r1; base += 256) {
        const int i0 = base + 4 * lane;
        int key[4];
        load_keys(f, i0, b, k, key);
        int before = 0, total = 0;
        bool hit[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            hit[c] = key[c] == j;
            unsigned long long m = __ballot(hit[c]);
            before += __popcll(m & below);
            total += __popcll(m);
        }
        int within = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (hit[c]) {
                perm[pos + before + within] = i0 + c;
                alpha_s[pos + before + within] = alpha[i0 + c];
                ++within;
            }
        }
        pos += total;
    }

    const int base_j = seg_start / P + j;
    const int np = (count + P - 1) / P;
    const int next_base = (j == k - 1) ? nslots : (seg_start + count) / P + j + 1;
    for (int q = tid; q < next_base - base_j; q += 1024) {
        const bool live = q < np;
        slot_row0[base_j + q] = live ? seg_start + q * P : 0;
        slot_len[base_j + q] = live ? min(P, count - q * P) : 0;
    }
    if (tid == 0) { sbase[j] = base_j; snum[j] = np; }
}

// ------------------------------------------------------------------------------------------------
// k_contract.  One wave per (slot, 512-column group); lane covers 8 consecutive columns.
template <typename TR> struct RowLoad;

template <> struct RowLoad<Bf16> {      // 8 columns = one 16-byte chunk
    uint4 v;
    __device__ __forceinline__ void load(const uint4* __restrict__ rowp, int ch, int mch) { v = ch < mch ? rowp[ch] : make_uint4(0, 0, 0, 0); }
    __device__ __forceinline__ void fma(float a, float (&acc)[8]) const {
        float e[8];
        Bf16::unpack(v, e);
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] = fmaf(a, e[q], acc[q]);
    }
    static __device__ __forceinline__ int chunk_of(int grp, int lane) { return grp * 64 + lane; }
    static __device__ __forceinline__ bool any(int ch, int mch) { return ch < mch; }
    static __device__ __forceinline__ bool second_half(int, int) { return true; }
};

template <> struct RowLoad<F32> {       // 8 columns = two 16-byte chunks
    uint4 v0, v1;
    __device__ __forceinline__ void load(const uint4* __restrict__ rowp, int ch, int mch) {
        v0 = ch < mch ? rowp[ch] : make_uint4(0, 0, 0, 0);
        v1 = ch + 1 < mch ? rowp[ch + 1] : make_uint4(0, 0, 0, 0);
    }
    __device__ __forceinline__ void fma(float a, float (&acc)[8]) const {
        acc[0] = fmaf(a, __uint_as_float(v0.x), acc[0]); acc[1] = fmaf(a, __uint_as_float(v0.y), acc[1]);
        acc[2] = fmaf(a, __uint_as_float(v0.z), acc[2]); acc[3] = fmaf(a, __uint_as_float(v0.w), acc[3]);
        acc[4] = fmaf(a, __uint_as_float(v1.x), acc[4]); acc[5] = fmaf(a, __uint_as_float(v1.y), acc[5]);
        acc[6] = fmaf(a, __uint_as_float(v1.z), acc[6]); acc[7] = fmaf(a, __uint_as_float(v1.w), acc[7]);
    }
    static __device__ __forceinline__ int chunk_of(int grp, int lane) { return 2 * (grp * 64 + lane); }
    static __device__ __forceinline__ bool any(int ch, int mch) { return ch < mch; }
    static __device__ __forceinline__ bool second_half(int ch, int mch) { return ch + 1 < mch; }
};

template <typename TR>
__global__ __launch_bounds__(64) void k_contract(const uint4* __restrict__ dY, const int32_t* __restrict__ perm,
                                                 const float* __restrict__ alpha_s, const int32_t* __restrict__ slot_row0,
                                                 const int32_t* __restrict__ slot_len, int mch, int m, int cg,
                                                 float* __restrict__ partial) {
    const int slot = blockIdx.x / cg, grp = blockIdx.x % cg;
    const int len = slot_len[slot];
    if (len == 0) return;
    const int row0 = slot_row0[slot];
    const int lane = threadIdx.x;
    const int ch = RowLoad<TR>::chunk_of(grp, lane);

    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.f;

    constexpr int U = 8;
    int r = 0;
    for (; r + U <= len; r += U) {
        RowLoad<TR> v[U];
        float a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int row = __builtin_amdgcn_readfirstlane(perm[row0 + r + u]);
            a[u] = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(alpha_s[row0 + r + u])));
            v[u].load(dY + size_t(row) * mch, ch, mch);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) v[u].fma(a[u], acc);
    }
    for (; r < len; ++r) {
        const int row = __builtin_amdgcn_readfirstlane(perm[row0 + r]);
        const float a = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(alpha_s[row0 + r])));
        RowLoad<TR> v;
        v.load(dY + size_t(row) * mch, ch, mch);
        v.fma(a, acc);
    }

    const int col = grp * 512 + lane * 8;
    if (col < m) {
        float4* dst = reinterpret_cast<float4*>(partial + size_t(slot) * m + col);
        dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        if (col + 4 < m) dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
}

// Btilde_j = sum of generator j's partial rows (only used by pamm_contract).
__global__ __launch_bounds__(256) void k_piece_sum(const float* __restrict__ partial, const int32_t* __restrict__ sbase,
                                                   const int32_t* __restrict__ snum, int m, float* __restrict__ Bt) {
    const int j = blockIdx.y;
    const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (c >= m) return;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    const int base = sbase[j], np = snum[j];
    for (int q = 0; q < np; ++q) {
        float4 v = *reinterpret_cast<const float4*>(partial + size_t(base + q) * m + c);
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    *reinterpret_cast<float4*>(Bt + size_t(j) * m + c) = s;
}

// ------------------------------------------------------------------------------------------------
// k_ctb: dW (n x m) = C^T (n x k) * Btilde (k x m).  Workgroup tile 128 x 128, 4 waves of 64 x 64,
// generators walked 32 at a time.  Both operands arrive with the generator index as the slow
// dimension, while the MFMA wants it contiguous per lane, so each stage is transposed on its way
// into LDS: At[l][j], Bt[c][j], rows padded by 16 bytes.
template <typename TR> struct CtbStage;

template <> struct CtbStage<Bf16> {
    static constexpr int kRowWords = 16 + 4;       // 32 bf16 + pad
    // A: thread -> (generator pair jp, group of 8 hidden indices lg)
    static __device__ __forceinline__ void stage_a(const uint4* __restrict__ C, int nch, int n, int k, int j0, int l0, int tid,
                                                   uint32_t* __restrict__ At) {
        const int jp = tid & 15, lg = tid >> 4;
        const int j = j0 + 2 * jp, l = l0 + 8 * lg;
        uint4 lo = make_uint4(0, 0, 0, 0), hi = lo;
        if (l < n) {
            if (j < k) lo = C[size_t(j) * nch + (l >> 3)];
            if (j + 1 < k) hi = C[size_t(j + 1) * nch + (l >> 3)];
        }
        const uint32_t a[4] = {lo.x, lo.y, lo.z, lo.w}, c[4] = {hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            uint32_t x = (e & 1) ? (a[e >> 1] >> 16) : (a[e >> 1] & 0xffffu);
            uint32_t y = (e & 1) ? (c[e >> 1] & 0xffff0000u) : (c[e >> 1] << 16);
            At[(8 * lg + e) * kRowWords + jp] = x | y;
        }
    }
    // B: thread -> two units of (generator pair jp, group of 4 columns cq)
    static __device__ __forceinline__ void stage_b(const float* __restrict__ partial, const int32_t* __restrict__ sbase,
                                                   const int32_t* __restrict__ snum, int m, int k, int j0, int c0, int tid,
                                                   uint32_t* __restrict__ Bt) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int unit = tid + 256 * h;
            const int jp = unit & 15, cq = unit >> 4;
            const int c = c0 + 4 * cq;
            float4 s[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                s[t] = make_float4(0.f, 0.f, 0.f, 0.f);
                const int j = j0 + 2 * jp + t;
                if (j < k && c < m) {
                    const int base = sbase[j], np = snum[j];
                    for (int q = 0; q < np; ++q) {
                        float4 v = *reinterpret_cast<const float4*>(partial + size_t(base + q) * m + c);
                        s[t].x += v.x; s[t].y += v.y; s[t].z += v.z; s[t].w += v.w;
                    }
                }
            }
            Bt[(4 * cq + 0) * kRowWords + jp] = pack_bf16(s[0].x, s[1].x);
            Bt[(4 * cq + 1) * kRowWords + jp] = pack_bf16(s[0].y, s[1].y);
            Bt[(4 * cq + 2) * kRowWords + jp] = pack_bf16(s[0].z, s[1].z);
            Bt[(4 * cq + 3) * kRowWords + jp] = pack_bf16(s[0].w, s[1].w);
        }
    }
};

template <> struct CtbStage<F32> {
    static constexpr int kRowWords = 32 + 4;       // 32 fp32 + pad
    // A: thread -> four units of (generator j, group of 4 hidden indices lq)
    static __device__ __forceinline__ void stage_a(const uint4* __restrict__ C, int nch, int n, int k, int j0, int l0, int tid,
                                                   uint32_t* __restrict__ At) {
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            const int unit = tid + 256 * h;
            const int jj = unit & 31, lq = unit >> 5;
            const int j = j0 + jj, l = l0 + 4 * lq;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (j < k && l < n) v = C[size_t(j) * nch + (l >> 2)];
            At[(4 * lq + 0) * kRowWords + jj] = v.x;
            At[(4 * lq + 1) * kRowWords + jj] = v.y;
            At[(4 * lq + 2) * kRowWords + jj] = v.z;
            At[(4 * lq + 3) * kRowWords + jj] = v.w;
        }
    }
    static __device__ __forceinline__ void stage_b(const float* __restrict__ partial, const int32_t* __restrict__ sbase,
                                                   const int32_t* __restrict__ snum, int m, int k, int j0, int c0, int tid,
                                                   uint32_t* __restrict__ Bt) {
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            const int unit = tid + 256 * h;
            const int jj = unit & 31, cq = unit >> 5;
            const int j = j0 + jj, c = c0 + 4 * cq;
            float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
            if (j < k && c < m) {
                const int base = sbase[j], np = snum[j];
                for (int q = 0; q < np; ++q) {
                    float4 v = *reinterpret_cast<const float4*>(partial + size_t(base + q) * m + c);
                    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
                }
            }
            Bt[(4 * cq + 0) * kRowWords + jj] = __float_as_uint(s.x);
            Bt[(4 * cq + 1) * kRowWords + jj] = __float_as_uint(s.y);
            Bt[(4 * cq + 2) * kRowWords + jj] = __float_as_uint(s.z);
            Bt[(4 * cq + 3) * kRowWords + jj] = __float_as_uint(s.w);
        }
    }
};

template <typename TR>
__global__ __launch_bounds__(256) void k_ctb(const uint4* __restrict__ C, const float* __restrict__ partial,
                                             const int32_t* __restrict__ sbase, const int32_t* __restrict__ snum, int n, int m,
                                             int k, int tiles_m, float* __restrict__ dW) {
    constexpr int RW = CtbStage<TR>::kRowWords;
    constexpr int CALLS = 32 / (2 * TR::kPerChunk);     // mma calls per 32-generator stage: 2 (bf16) or 4 (fp32)
    __shared__ __attribute__((aligned(16))) uint32_t At[128 * RW];
    __shared__ __attribute__((aligned(16))) uint32_t Bt[128 * RW];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 31, g = lane >> 5;
    const int wy = wave >> 1, wx = wave & 1;
    const int l0 = (blockIdx.x / tiles_m) * 128, c0 = (blockIdx.x % tiles_m) * 128;
    const int nch = n / TR::kPerChunk;

    f32x16_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int bq = 0; bq < 2; ++bq)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][bq][i] = 0.f;

    for (int j0 = 0; j0 < k; j0 += 32) {
        __syncthreads();
        CtbStage<TR>::stage_a(C, nch, n, k, j0, l0, tid, At);
        CtbStage<TR>::stage_b(partial, sbase, snum, m, k, j0, c0, tid, Bt);
        __syncthreads();
#pragma unroll
        for (int t = 0; t < CALLS; ++t) {
            uint4 a[2], bq[2];
#pragma unroll
            for (int fa = 0; fa < 2; ++fa)
                a[fa] = *reinterpret_cast<const uint4*>(&At[(wy * 64 + 32 * fa + r) * RW + 4 * (2 * t + g)]);
#pragma unroll
            for (int fb = 0; fb < 2; ++fb)
                bq[fb] = *reinterpret_cast<const uint4*>(&Bt[(wx * 64 + 32 * fb + r) * RW + 4 * (2 * t + g)]);
#pragma unroll
            for (int fa = 0; fa < 2; ++fa)
#pragma unroll
                for (int fb = 0; fb < 2; ++fb) TR::mma(a[fa], bq[fb], acc[fa][fb]);
        }
    }

#pragma unroll
    for (int fa = 0; fa < 2; ++fa)
#pragma unroll
        for (int fb = 0; fb < 2; ++fb) {
            const int c = c0 + wx * 64 + 32 * fb + r;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int l = l0 + wy * 64 + 32 * fa + 8 * (i >> 2) + 4 * g + (i & 3);
                if (l < n && c < m) dW[size_t(l) * m + c] = acc[fa][fb][i];
            }
        }
}

// ------------------------------------------------------------------------------------------------ host side

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct GradBuffers {
    int32_t *perm, *row0, *len, *sbase, *snum;
    float *alpha_s, *partial;
};

static GradBuffers carve(const GradPlan& pl, char* ws) {
    GradBuffers g;
    g.perm = reinterpret_cast<int32_t*>(ws + pl.off_perm);
    g.alpha_s = reinterpret_cast<float*>(ws + pl.off_alpha);
    g.row0 = reinterpret_cast<int32_t*>(ws + pl.off_row0);
    g.len = reinterpret_cast<int32_t*>(ws + pl.off_len);
    g.sbase = reinterpret_cast<int32_t*>(ws + pl.off_sbase);
    g.snum = reinterpret_cast<int32_t*>(ws + pl.off_snum);
    g.partial = reinterpret_cast<float*>(ws + pl.off_partial);
    return g;
}

template <typename TR>
static void launch_group_contract(const GradPlan& pl, const GradBuffers& g, const int32_t* f, const float* alpha, const void* dY,
                                  int b, int k, int m, hipStream_t s) {
    {
        ScopedSpan span(kGroup, s);
        hipLaunchKernelGGL(k_group, dim3(k), dim3(1024), 0, s, f, alpha, b, k, pl.piece_rows, int(pl.nslots), g.perm, g.alpha_s,
                           g.row0, g.len, g.sbase, g.snum);
    }
    const int mch = m / TR::kPerChunk;
    {
        ScopedSpan span(kContract, s);
        hipLaunchKernelGGL((k_contract<TR>), dim3((unsigned)(pl.nslots * pl.col_groups)), dim3(64), 0, s, (const uint4*)dY, g.perm,
                           g.alpha_s, g.row0, g.len, mch, m, pl.col_groups, g.partial);
    }
}

}  // namespace pamm

using namespace pamm;

extern "C" pamm_status pamm_contract(const int32_t* f, const float* alpha, const void* dY, int64_t b, int64_t k, int64_t m,
                                     pamm_dtype dt, float* Btilde, void* ws, size_t ws_bytes, void* stream) {
    GradPlan pl;
    pamm_status st = plan_grad(b, per_chunk(dtype_ok(dt) ? dt : PAMM_F32), k, m, dt, &pl);   // n does not enter the layout
    if (st != PAMM_OK) return st;
    if (k > b) return PAMM_ERR_INVALID_ARG;
    if (!f || !alpha || !dY || !Btilde) return PAMM_ERR_INVALID_ARG;
    if (!aligned16(f) || !aligned16(alpha) || !aligned16(dY) || !aligned16(Btilde)) return PAMM_ERR_INVALID_ARG;
    if (!ws || ws_bytes < pl.total) return PAMM_ERR_WORKSPACE;
    if (!aligned16(ws)) return PAMM_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    GradBuffers g = carve(pl, (char*)ws);
    if (dt == PAMM_BF16) launch_group_contract<Bf16>(pl, g, f, alpha, dY, int(b), int(k), int(m), s);
    else launch_group_contract<F32>(pl, g, f, alpha, dY, int(b), int(k), int(m), s);
    {
        ScopedSpan span(kPieceSum, s);
        hipLaunchKernelGGL(k_piece_sum, dim3((unsigned)((m / 4 + 255) / 256), (unsigned)k), dim3(256), 0, s, g.partial, g.sbase,
                           g.snum, int(m), Btilde);
    }
    return hipGetLastError() == hipSuccess ? PAMM_OK : PAMM_ERR_DEVICE;
}

extern "C" pamm_status pamm_grad(const void* C, const int32_t* f, const float* alpha, const void* dY, int64_t b, int64_t n,
                                 int64_t k, int64_t m, pamm_dtype dt, float* dW, void* ws, size_t ws_bytes, void* stream) {
    GradPlan pl;
    pamm_status st = plan_grad(b, n, k, m, dt, &pl);
    if (st != PAMM_OK) return st;
    if (k > b) return PAMM_ERR_INVALID_ARG;
    if (!C || !f || !alpha || !dY || !dW) return PAMM_ERR_INVALID_ARG;
    if (!aligned16(C) || !aligned16(f) || !aligned16(alpha) || !aligned16(dY) || !aligned16(dW)) return PAMM_ERR_INVALID_ARG;
    if (!ws || ws_bytes < pl.total) return PAMM_ERR_WORKSPACE;
    if (!aligned16(ws)) return PAMM_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    GradBuffers g = carve(pl, (char*)ws);
    const int tiles_n = int((n + 127) / 128), tiles_m = int((m + 127) / 128);
    if (dt == PAMM_BF16) {
        launch_group_contract<Bf16>(pl, g, f, alpha, dY, int(b), int(k), int(m), s);
        ScopedSpan span(kCtb, s);
        hipLaunchKernelGGL((k_ctb<Bf16>), dim3((unsigned)(tiles_n * tiles_m)), dim3(256), 0, s, (const uint4*)C, g.partial, g.sbase,
                           g.snum, int(n), int(m), int(k), tiles_m, dW);
    } else {
        launch_group_contract<F32>(pl, g, f, alpha, dY, int(b), int(k), int(m), s);
        ScopedSpan span(kCtb, s);
        hipLaunchKernelGGL((k_ctb<F32>), dim3((unsigned)(tiles_n * tiles_m)), dim3(256), 0, s, (const uint4*)C, g.partial, g.sbase,
                           g.snum, int(n), int(m), int(k), tiles_m, dW);
    }
    return hipGetLastError() == hipSuccess ? PAMM_OK : PAMM_ERR_DEVICE;
}
