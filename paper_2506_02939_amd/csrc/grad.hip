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
//
// The sorted list (perm, alpha_s, key_s) is later cut into chunks of P consecutive positions; a
// "piece" is a maximal run of one generator inside one chunk and is numbered chunk + generator.
// Piece numbers are unique, increase along the list and stay below ceil(b/P) + k.  Generator j owns
// the pieces [seg_start_j / P + j, (seg_end_j - 1) / P + j].
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
                                                int P, int32_t* __restrict__ perm, float* __restrict__ alpha_s,
                                                int32_t* __restrict__ key_s, int32_t* __restrict__ sbase,
                                                int32_t* __restrict__ snum) {
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

    if (s_eq[wave] > 0) {                  // wave-uniform: most waves hold no row of this generator when k is large
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
                    key_s[pos + before + within] = j;
                    ++within;
                }
            }
            pos += total;
        }
    }
    if (tid == 0) {
        sbase[j] = seg_start / P + j;
        snum[j] = count > 0 ? (seg_start + count - 1) / P - seg_start / P + 1 : 0;
    }
}

// ------------------------------------------------------------------------------------------------
// k_contract.  One wave per (chunk of P list positions, 512-column group); lane covers 8 consecutive
// columns.  Every wave moves the same number of bytes, whatever the sizes of the generators' lists.
// When the generator changes inside a chunk the running sums are written out as one piece and reset.
template <typename TR> struct RowLoad;

template <> struct RowLoad<Bf16> {      // 8 columns = one 16-byte chunk
    u32x4_t v;
    static constexpr int kGroup = 8;     // rows fetched per group
    __device__ __forceinline__ void load(const u32x4_t* __restrict__ rowp, int ch, int) { v = rowp[ch]; }
    __device__ __forceinline__ void fma(float a, float (&acc)[8]) const {
        float e[8];
        Bf16::unpack(v, e);
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] = fmaf(a, e[q], acc[q]);
    }
    // chunk index of this lane, clamped into the row (lanes past the last column load valid data and store nothing)
    static __device__ __forceinline__ int chunk_of(int grp, int lane, int mch) { return min(grp * 64 + lane, mch - 1); }
};

template <> struct RowLoad<F32> {       // 8 columns = two 16-byte chunks
    u32x4_t v0, v1;
    static constexpr int kGroup = 4;
    __device__ __forceinline__ void load(const u32x4_t* __restrict__ rowp, int ch, int mch) { v0 = rowp[ch]; v1 = rowp[min(ch + 1, mch - 1)]; }
    __device__ __forceinline__ void fma(float a, float (&acc)[8]) const {
        acc[0] = fmaf(a, __uint_as_float(v0.x), acc[0]); acc[1] = fmaf(a, __uint_as_float(v0.y), acc[1]);
        acc[2] = fmaf(a, __uint_as_float(v0.z), acc[2]); acc[3] = fmaf(a, __uint_as_float(v0.w), acc[3]);
        acc[4] = fmaf(a, __uint_as_float(v1.x), acc[4]); acc[5] = fmaf(a, __uint_as_float(v1.y), acc[5]);
        acc[6] = fmaf(a, __uint_as_float(v1.z), acc[6]); acc[7] = fmaf(a, __uint_as_float(v1.w), acc[7]);
    }
    static __device__ __forceinline__ int chunk_of(int grp, int lane, int mch) { return min(2 * (grp * 64 + lane), mch - 1); }
};

template <typename TR>
__global__ __launch_bounds__(64) void k_contract(const u32x4_t* __restrict__ dY, const int32_t* __restrict__ perm,
                                                 const float* __restrict__ alpha_s, const int32_t* __restrict__ key_s, int b,
                                                 int P, int mch, int m, int cg, float* __restrict__ partial) {
    const int chunk = blockIdx.x / cg, grp = blockIdx.x % cg;
    const int s0 = chunk * P;
    const int s1 = min(b, s0 + P);
    const int lane = threadIdx.x;
    const int ch = RowLoad<TR>::chunk_of(grp, lane, mch);
    const int col = grp * 512 + lane * 8;

    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.f;
    int cur = __builtin_amdgcn_readfirstlane(key_s[s0]);

    auto flush = [&](int key) {
        if (col < m) {
            float4* dst = reinterpret_cast<float4*>(partial + size_t(chunk + key) * m + col);
            dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
            if (col + 4 < m) dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] = 0.f;
    };

    // Rows are fetched in groups of U; the next group's loads are issued before the current group is consumed.
    // Positions past the end of the chunk re-read its last row with weight 0 (no guard around the loads).
    constexpr int U = RowLoad<TR>::kGroup;
    auto issue = [&](RowLoad<TR> (&v)[U], float (&a)[U], int (&key)[U], int s) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int pos = min(s + u, s1 - 1);
            const int row = __builtin_amdgcn_readfirstlane(perm[pos]);
            const float al = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(alpha_s[pos])));
            key[u] = __builtin_amdgcn_readfirstlane(key_s[pos]);
            a[u] = (s + u < s1) ? al : 0.f;
            v[u].load(dY + size_t(row) * mch, ch, mch);
        }
    };
    auto consume = [&](const RowLoad<TR> (&v)[U], const float (&a)[U], const int (&key)[U]) {
        if (key[0] == cur && key[U - 1] == cur) {          // the list is sorted: the whole group belongs to `cur`
#pragma unroll
            for (int u = 0; u < U; ++u) v[u].fma(a[u], acc);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (key[u] != cur) { flush(cur); cur = key[u]; }
                v[u].fma(a[u], acc);
            }
        }
    };
    RowLoad<TR> va[U], vb[U];
    float aa[U], ab[U];
    int ka[U], kb[U];
    issue(va, aa, ka, s0);
    for (int s = s0; s < s1; s += 2 * U) {
        const bool hb = s + U < s1, ha = s + 2 * U < s1;        // uniform
        if (hb) issue(vb, ab, kb, s + U);
        consume(va, aa, ka);
        if (ha) issue(va, aa, ka, s + 2 * U);
        if (hb) consume(vb, ab, kb);
    }
    flush(cur);
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
// k_prep: puts both operands of C^T Btilde into the layout the MFMA wants, generator index contiguous:
//   Bt[c][j] = Btilde_j[c] = sum of generator j's pieces (rounded once to bf16 for bf16 inputs), Ct[l][j] = C_j[l],
// rows padded with zeros to KP generators (a whole number of MFMA steps).  One thread per 16-byte chunk.
template <typename TR> struct PackChunk;
template <> struct PackChunk<Bf16> {
    static __device__ __forceinline__ u32x4_t from_floats(const float (&v)[8]) {
        return u32x4_t{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
    }
    static __device__ __forceinline__ u32x4_t gather_c(const void* C, size_t n, int l, int j0, int k) {
        const uint16_t* c = static_cast<const uint16_t*>(C);
        uint32_t e[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) e[q] = (j0 + q < k) ? uint32_t(c[size_t(j0 + q) * n + l]) : 0u;
        return u32x4_t{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
    }
};
template <> struct PackChunk<F32> {
    static __device__ __forceinline__ u32x4_t from_floats(const float (&v)[4]) {
        return u32x4_t{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
    }
    static __device__ __forceinline__ u32x4_t gather_c(const void* C, size_t n, int l, int j0, int k) {
        const uint32_t* c = static_cast<const uint32_t*>(C);
        uint32_t e[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) e[q] = (j0 + q < k) ? c[size_t(j0 + q) * n + l] : 0u;
        return u32x4_t{e[0], e[1], e[2], e[3]};
    }
};

template <typename TR>
__global__ __launch_bounds__(256) void k_prep(const void* __restrict__ C, const float* __restrict__ partial,
                                              const int32_t* __restrict__ sbase, const int32_t* __restrict__ snum, int n, int m,
                                              int k, int KC, int blocks_m, u32x4_t* __restrict__ Ct, u32x4_t* __restrict__ Bt) {
    constexpr int JPC = TR::kPerChunk;
    const int jg = blockIdx.y, j0 = jg * JPC;
    if (int(blockIdx.x) < blocks_m) {
        const int c = blockIdx.x * 256 + threadIdx.x;
        if (c >= m) return;
        float v[JPC];
#pragma unroll
        for (int q = 0; q < JPC; ++q) {
            float s = 0.f;
            const int j = j0 + q;
            if (j < k) {                                   // uniform
                const int base = sbase[j], np = snum[j];
                for (int t = 0; t < np; ++t) s += partial[size_t(base + t) * m + c];
            }
            v[q] = s;
        }
        Bt[size_t(c) * KC + jg] = PackChunk<TR>::from_floats(v);
    } else {
        const int l = (blockIdx.x - blocks_m) * 256 + threadIdx.x;
        if (l >= n) return;
        Ct[size_t(l) * KC + jg] = PackChunk<TR>::gather_c(C, size_t(n), l, j0, k);
    }
}

// ------------------------------------------------------------------------------------------------
// k_ctb: dW (n x m) = C^T (n x k) * Btilde (k x m).  Workgroup tile 128 x 128, 4 waves of 64 x 64.  Both
// operands come from k_prep with the generator index contiguous, so every MFMA fragment is one 16-byte
// load per lane straight from L2/L1 (both operands together are a few MiB): no LDS, no barriers.  The
// kernel is bound by writing dW.
template <typename TR>
__global__ __launch_bounds__(256) void k_ctb(const u32x4_t* __restrict__ Ct, const u32x4_t* __restrict__ Bt, int n, int m, int KC,
                                             int tiles_m, float* __restrict__ dW) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 31, g = lane >> 5;
    const int wy = wave >> 1, wx = wave & 1;
    const int l0 = (blockIdx.x / tiles_m) * 128 + wy * 64, c0 = (blockIdx.x % tiles_m) * 128 + wx * 64;

    const u32x4_t* arow[2];
    const u32x4_t* brow[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        arow[q] = Ct + size_t(min(l0 + 32 * q + r, n - 1)) * KC + g;
        brow[q] = Bt + size_t(min(c0 + 32 * q + r, m - 1)) * KC + g;
    }
    f32x16_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int bq = 0; bq < 2; ++bq)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][bq][i] = 0.f;

#pragma unroll 4
    for (int t = 0; t < KC; t += 2) {          // one mma call takes chunk t + g from every lane
        u32x4_t a[2], bq[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) { a[q] = arow[q][t]; bq[q] = brow[q][t]; }
#pragma unroll
        for (int fa = 0; fa < 2; ++fa)
#pragma unroll
            for (int fb = 0; fb < 2; ++fb) TR::mma(a[fa], bq[fb], acc[fa][fb]);
    }

#pragma unroll
    for (int fa = 0; fa < 2; ++fa)
#pragma unroll
        for (int fb = 0; fb < 2; ++fb) {
            const int c = c0 + 32 * fb + r;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int l = l0 + 32 * fa + 8 * (i >> 2) + 4 * g + (i & 3);
                if (l < n && c < m) dW[size_t(l) * m + c] = acc[fa][fb][i];
            }
        }
}

// ------------------------------------------------------------------------------------------------ host side

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct GradBuffers {
    int32_t *perm, *key, *sbase, *snum;
    float *alpha_s, *partial;
    u32x4_t *ct, *bt;
};

static GradBuffers carve(const GradPlan& pl, char* ws) {
    GradBuffers g;
    g.perm = reinterpret_cast<int32_t*>(ws + pl.off_perm);
    g.alpha_s = reinterpret_cast<float*>(ws + pl.off_alpha);
    g.key = reinterpret_cast<int32_t*>(ws + pl.off_key);
    g.sbase = reinterpret_cast<int32_t*>(ws + pl.off_sbase);
    g.snum = reinterpret_cast<int32_t*>(ws + pl.off_snum);
    g.partial = reinterpret_cast<float*>(ws + pl.off_partial);
    g.ct = reinterpret_cast<u32x4_t*>(ws + pl.off_ct);
    g.bt = reinterpret_cast<u32x4_t*>(ws + pl.off_bt);
    return g;
}

template <typename TR>
static void launch_group_contract(const GradPlan& pl, const GradBuffers& g, const int32_t* f, const float* alpha, const void* dY,
                                  int b, int k, int m, hipStream_t s) {
    {
        ScopedSpan span(kGroup, s);
        hipLaunchKernelGGL(k_group, dim3(k), dim3(1024), 0, s, f, alpha, b, k, pl.piece_rows, g.perm, g.alpha_s, g.key, g.sbase,
                           g.snum);
    }
    const int mch = m / TR::kPerChunk;
    {
        ScopedSpan span(kContract, s);
        hipLaunchKernelGGL((k_contract<TR>), dim3((unsigned)(pl.chunks * pl.col_groups)), dim3(64), 0, s, (const u32x4_t*)dY, g.perm,
                           g.alpha_s, g.key, b, pl.piece_rows, mch, m, pl.col_groups, g.partial);
    }
}

template <typename TR>
static void launch_prep_ctb(const GradPlan& pl, const GradBuffers& g, const void* C, int n, int m, int k, float* dW, hipStream_t s) {
    const int KC = int(pl.kpad) / TR::kPerChunk;
    const int blocks_m = (m + 255) / 256, blocks_n = (n + 255) / 256;
    {
        ScopedSpan span(kPrep, s);
        hipLaunchKernelGGL((k_prep<TR>), dim3((unsigned)(blocks_m + blocks_n), (unsigned)KC), dim3(256), 0, s, C, g.partial, g.sbase,
                           g.snum, n, m, k, KC, blocks_m, g.ct, g.bt);
    }
    const int tiles_n = (n + 127) / 128, tiles_m = (m + 127) / 128;
    {
        ScopedSpan span(kCtb, s);
        hipLaunchKernelGGL((k_ctb<TR>), dim3((unsigned)(tiles_n * tiles_m)), dim3(256), 0, s, g.ct, g.bt, n, m, KC, tiles_m, dW);
    }
}

}  // namespace pamm

using namespace pamm;

extern "C" pamm_status pamm_contract(const int32_t* f, const float* alpha, const void* dY, int64_t b, int64_t k, int64_t m,
                                     pamm_dtype dt, float* Btilde, void* ws, size_t ws_bytes, void* stream) {
    GradPlan pl;
    pamm_status st = plan_grad(b, per_chunk(dtype_ok(dt) ? dt : PAMM_F32), k, m, dt, &pl);   // n does not enter what is used here
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
    if (dt == PAMM_BF16) {
        launch_group_contract<Bf16>(pl, g, f, alpha, dY, int(b), int(k), int(m), s);
        launch_prep_ctb<Bf16>(pl, g, C, int(n), int(m), int(k), dW, s);
    } else {
        launch_group_contract<F32>(pl, g, f, alpha, dY, int(b), int(k), int(m), s);
        launch_prep_ctb<F32>(pl, g, C, int(n), int(m), int(k), dW, s);
    }
    return hipGetLastError() == hipSuccess ? PAMM_OK : PAMM_ERR_DEVICE;
}
