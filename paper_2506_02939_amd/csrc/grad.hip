// pamm_grad / pamm_grad_eps / pamm_grad_out / pamm_contract: Alg. 1, procedure ApproxMM.
//
// Launches on the caller's stream:
//   grouping    stable grouping of the rows by f(i) into one sorted list of 16-byte entries, cut into chunks of P
//               positions: a counting sort (k_sort_one for b <= 16384, k_hist + k_scatter above that) for
//               k <= 2048, one workgroup per generator (k_group_regs / k_group_stream) for larger k
//   k_contract  streams dY once: one wave per (chunk, 512 columns) sums alpha_i * dY_i in registers, in list
//               order, and writes one fp32 partial row per piece.  No atomics, no LDS; bit-reproducible.
//   k_prep      Btilde_j = sum of generator j's partial rows (times beta); both operands of the product laid out
//               with the generator index contiguous
//   k_ctb       dW = C^T Btilde on the matrix cores
#include <hip/hip_runtime.h>

#include <atomic>
#include <type_traits>

#include "pamm_device.h"
#include "pamm_plan.h"
#include "pamm_profile.h"
#include "pamm_tile256.h"

namespace pamm {

// ------------------------------------------------------------------------------------------------
// k_group.  grid = k, 1024 threads.  Every workgroup reads all of f twice (f is b int32: it stays in
// L2): pass 1 counts rows with key < j (start of generator j's list) and key == j per wave, pass 2
// compacts the matching row numbers with ballots, which keeps them in increasing order.
//
// The sorted list holds one 16-byte entry per row with a non-zero weight: {row number, alpha_i (bits), generator, 0}.
// Rows with alpha_i = 0 (dropped by the neighbourhood condition, or orthogonal to their generator) add nothing to
// Btilde and are left out, so their rows of dY are never read.  The list of L entries is later cut into chunks of P
// consecutive positions, P chosen on the device from L so that every CU gets one chunk; a "piece" is a maximal
// run of one generator inside one chunk and is numbered chunk + generator.  Piece numbers are unique, increase
// along the list and stay below the number of chunks + k.  Generator j owns the pieces
// [seg_start_j / P + j, (seg_end_j - 1) / P + j].
__device__ __forceinline__ void load_keys(const int32_t* __restrict__ f, const float* __restrict__ alpha, int i0, int b, int k,
                                          int (&key)[4]) {
    float w[4];
    if (i0 + 3 < b) {
        const int4 v = *reinterpret_cast<const int4*>(f + i0);
        const float4 a = *reinterpret_cast<const float4*>(alpha + i0);
        key[0] = v.x; key[1] = v.y; key[2] = v.z; key[3] = v.w;
        w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w;
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            key[c] = (i0 + c < b) ? f[i0 + c] : -1;
            w[c] = (i0 + c < b) ? alpha[i0 + c] : 0.f;
        }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const bool in = i0 + c < b && w[c] != 0.f;
        int v = key[c];
        v = v < 0 ? 0 : (v >= k ? k - 1 : v);
        key[c] = in ? v : k;            // k = "no row": larger than every generator number
    }
}

// One row's key (as load_keys) and weight; rows past the end count as "no row".
__device__ __forceinline__ int load_key(const int32_t* __restrict__ f, const float* __restrict__ alpha, int i, int b, int k, float& w) {
    const bool in = i < b;
    const int ii = in ? i : b - 1;
    int v = f[ii];
    w = alpha[ii];
    v = v < 0 ? 0 : (v >= k ? k - 1 : v);
    return (in && w != 0.f) ? v : k;
}

// The lanes of the wave whose key equals this lane's (this lane included): the key's bits are peeled off one ballot
// at a time, so the cost does not depend on how many different keys the wave holds.  nbits covers the values 0..k.
__device__ __forceinline__ unsigned long long lanes_with_my_key(int key, int nbits) {
    unsigned long long same = ~0ull;
    for (int bit = 0; bit < nbits; ++bit) {
        const bool set = (key >> bit) & 1;
        const unsigned long long bal = __ballot(set);
        same &= set ? bal : ~bal;
    }
    return same;
}

// Position of a row inside its generator's part of the sorted list, for the 64 rows (one per lane, in increasing
// row order) that a wave places at a time: `ctr` points at the wave's own LDS counter for this lane's generator
// (rows of the generator the wave has placed so far, on top of the rows of earlier waves and slices).  Equal keys
// take consecutive positions in lane order, so together with the order of the calls the rows of one generator
// stay in increasing row order: the sort is stable by construction, no atomic decides an order.
__device__ __forceinline__ int stable_slot(int* ctr, bool live, int key, int nbits) {
    const unsigned long long same = lanes_with_my_key(key, nbits);
    const int lane = threadIdx.x & 63;
    const int rank = __popcll(same & ((1ull << lane) - 1ull));
    int old = 0;
    if (live) old = *ctr;                                   // every lane of the group reads before its leader writes
    wave_lds_sync();
    if (live && rank == 0) *ctr = old + __popcll(same);
    wave_lds_sync();
    return old + rank;
}

// What the grouping kernels leave for k_contract: hdr[0] = L, entries in the list; hdr[1] = P, positions per chunk.

// Chunk size for a list of L entries: one chunk per CU and workgroup column (256 CUs), a multiple of 16, at most 4096;
// p_fixed > 0 overrides (tuning).  The host sizes the partial-row buffer for the largest chunk count this can give.
__device__ __forceinline__ int piece_rows_for(int L, int wg_cols, int p_fixed) {
    if (p_fixed > 0) return p_fixed;
    long long P = ((long long)L * wg_cols + 255) / 256;
    P = (P + 15) / 16 * 16;
    return int(P < 16 ? 16 : (P > 4096 ? 4096 : P));
}

__device__ __forceinline__ u32x4_t list_entry(int row, float a, int key) {
    return u32x4_t{uint32_t(row), __float_as_uint(a), uint32_t(key), 0u};
}

// Entries L .. roundup(L,16)-1 of the sorted list repeat the last real entry with weight 0 (a row that is read
// anyway, so the padding touches no other row of dY).  Written by whoever writes entry L-1.
__device__ __forceinline__ void pad_list(u32x4_t* __restrict__ list, int L, int last_row, int last_key) {
    for (int q = L; q < (L + 15) / 16 * 16; ++q) list[q] = list_entry(last_row, 0.f, last_key);
}

// Generic version: two passes over f from L2, any b.
__global__ __launch_bounds__(1024) void k_group_stream(const int32_t* __restrict__ f, const float* __restrict__ alpha, int b, int k,
                                                       int wg_cols, int p_fixed, u32x4_t* __restrict__ list,
                                                       int32_t* __restrict__ sbase, int32_t* __restrict__ snum,
                                                       int32_t* __restrict__ hdr) {
    const int j = blockIdx.x;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const long long per_wave = (((long long)b + 15) / 16 + 255) / 256 * 256;
    const long long r0l = per_wave * wave;
    const int r0 = r0l < b ? int(r0l) : b;
    const int r1 = (r0l + per_wave) < b ? int(r0l + per_wave) : b;

    int lt = 0, eq = 0, live = 0;
    for (int base = r0; base < r1; base += 256) {
        int key[4];
        load_keys(f, alpha, base + 4 * lane, b, k, key);
#pragma unroll
        for (int c = 0; c < 4; ++c) { lt += key[c] < j; eq += key[c] == j; live += key[c] < k; }
    }
    lt = wave_sum(lt);
    eq = wave_sum(eq);
    live = wave_sum(live);
    __shared__ int s_lt[16], s_eq[16], s_live[16];
    if (lane == 0) { s_lt[wave] = lt; s_eq[wave] = eq; s_live[wave] = live; }
    __syncthreads();
    int seg_start = 0, count = 0, woff = 0, L = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        seg_start += s_lt[w];
        woff += (w < wave) ? s_eq[w] : 0;
        count += s_eq[w];
        L += s_live[w];
    }
    const int P = piece_rows_for(L, wg_cols, p_fixed);

    if (s_eq[wave] > 0) {                  // wave-uniform: most waves hold no row of this generator when k is large
        int pos = seg_start + woff;
        const unsigned long long below = (1ull << lane) - 1ull;
        for (int base = r0; base < r1; base += 256) {
            const int i0 = base + 4 * lane;
            int key[4];
            load_keys(f, alpha, i0, b, k, key);
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
                    list[pos + before + within] = list_entry(i0 + c, alpha[i0 + c], j);
                    if (pos + before + within == L - 1) pad_list(list, L, i0 + c, j);
                    ++within;
                }
            }
            pos += total;
        }
    }
    if (tid == 0) {
        sbase[j] = seg_start / P + j;
        snum[j] = count > 0 ? (seg_start + count - 1) / P - seg_start / P + 1 : 0;
        if (j == 0) { hdr[0] = L; hdr[1] = P; }
    }
}

// Version for b <= 16 waves * NV * 256 rows (NV <= 16, i.e. b <= 65536): every lane keeps its 4*NV keys in
// registers, so f is read once and both passes run out of registers.
template <int NV>
__global__ __launch_bounds__(1024) void k_group_regs(const int32_t* __restrict__ f, const float* __restrict__ alpha, int b, int k,
                                                     int wg_cols, int p_fixed, u32x4_t* __restrict__ list,
                                                     int32_t* __restrict__ sbase, int32_t* __restrict__ snum,
                                                     int32_t* __restrict__ hdr) {
    const int j = blockIdx.x;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int r0 = wave * (NV * 256);
    int key[NV][4];
#pragma unroll
    for (int v = 0; v < NV; ++v) load_keys(f, alpha, r0 + v * 256 + 4 * lane, b, k, key[v]);

    int lt = 0, eq = 0, live = 0;
#pragma unroll
    for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int c = 0; c < 4; ++c) { lt += key[v][c] < j; eq += key[v][c] == j; live += key[v][c] < k; }
    lt = wave_sum(lt);
    eq = wave_sum(eq);
    live = wave_sum(live);
    __shared__ int s_lt[16], s_eq[16], s_live[16];
    if (lane == 0) { s_lt[wave] = lt; s_eq[wave] = eq; s_live[wave] = live; }
    __syncthreads();
    int seg_start = 0, count = 0, woff = 0, L = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        seg_start += s_lt[w];
        woff += (w < wave) ? s_eq[w] : 0;
        count += s_eq[w];
        L += s_live[w];
    }
    const int P = piece_rows_for(L, wg_cols, p_fixed);

    if (eq > 0) {                          // wave-uniform
        int pos = seg_start + woff;
        const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int i0 = r0 + v * 256 + 4 * lane;
            int before = 0, total = 0;
            bool hit[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                hit[c] = key[v][c] == j;
                unsigned long long m = __ballot(hit[c]);
                before += __popcll(m & below);
                total += __popcll(m);
            }
            if (total > 0) {               // wave-uniform
                int within = 0;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (hit[c]) {
                        list[pos + before + within] = list_entry(i0 + c, alpha[i0 + c], j);
                        if (pos + before + within == L - 1) pad_list(list, L, i0 + c, j);
                        ++within;
                    }
                }
                pos += total;
            }
        }
    }
    if (tid == 0) {
        sbase[j] = seg_start / P + j;
        snum[j] = count > 0 ? (seg_start + count - 1) / P - seg_start / P + 1 : 0;
        if (j == 0) { hdr[0] = L; hdr[1] = P; }
    }
}

// ------------------------------------------------------------------------------------------------
// Grouping in O(b) for k <= 2048: a counting sort over slices of 4*NT rows (NT threads per workgroup).
//   k_hist     one workgroup per slice: histogram of the slice's keys (LDS atomics), written to table[slice][j]
//   k_scatter  one workgroup per slice: start of every generator's list (sum over all slices, scanned over j), plus
//              the rows of earlier slices, plus the rows of earlier waves of this slice; then every row takes its
//              position behind the rows of its generator that precede it and writes its 16-byte list entry.
// Wave w of a slice owns its rows [256 w, 256 w + 256) and places them 64 at a time in increasing order; equal keys
// inside such a group of 64 take consecutive positions in lane order (stable_slot), so the rows of one generator stay
// in increasing row order whatever the hardware does: the list, and every sum formed from it, is the same on every
// call, and the same as the per-generator grouping kernels produce.
constexpr int kScatterMaxK = 2048;     // (NT/64 + 2) * k ints of LDS

template <int NT>
__global__ __launch_bounds__(NT) void k_hist(const int32_t* __restrict__ f, const float* __restrict__ alpha, int b, int k,
                                             int32_t* __restrict__ table) {
    extern __shared__ int hist[];
    const int tid = threadIdx.x;
    int key[4];
    load_keys(f, alpha, blockIdx.x * (4 * NT) + 4 * tid, b, k, key);
    for (int j = tid; j < k; j += NT) hist[j] = 0;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 4; ++c)
        if (key[c] < k) atomicAdd(&hist[key[c]], 1);
    __syncthreads();
    for (int j = tid; j < k; j += NT) table[size_t(blockIdx.x) * k + j] = hist[j];
}

template <int NT>
__global__ __launch_bounds__(NT) void k_scatter(const int32_t* __restrict__ f, const float* __restrict__ alpha, int b, int k,
                                                int wg_cols, int p_fixed, int nslices, const int32_t* __restrict__ table,
                                                u32x4_t* __restrict__ list, int32_t* __restrict__ sbase,
                                                int32_t* __restrict__ snum, int32_t* __restrict__ hdr) {
    constexpr int NWV = NT / 64;
    extern __shared__ int lds[];
    int* wh = lds;                 // [NWV][k] per-wave counts, later per-wave next free position inside the generator's list
    int* tot = lds + NWV * k;      // [k]      rows per generator (whole batch), later start of the generator's list
    int* bef = tot + k;            // [k]      rows per generator in earlier slices
    __shared__ int wsum[NWV];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int slice = blockIdx.x;

    // every global load of the kernel is issued up front (keys, weights, this thread's share of the table), so the
    // kernel pays one memory latency, not one per phase
    int key[4];
    float al[4];
    const int i0 = slice * (4 * NT) + 256 * wave + lane;      // wave w owns rows [256 w, 256 w + 256) of the slice; slot c: + 64 c
#pragma unroll
    for (int c = 0; c < 4; ++c) key[c] = load_key(f, alpha, i0 + 64 * c, b, k, al[c]);
    // rows of every generator in earlier slices / in all slices: column sums of the table, taken in parallel by all
    // threads: `strips` threads per generator when there are fewer generators than threads, each summing every
    // strips-th slice; otherwise every thread sums whole columns for the generators tid, tid + NT, ...
    constexpr int GPT = (kScatterMaxK + NT - 1) / NT;          // generators per thread at most
    const int strips = k <= NT ? NT / k : 1;
    int before[GPT], total[GPT];
#pragma unroll
    for (int h = 0; h < GPT; ++h) {
        before[h] = total[h] = 0;
        const int j = h * NT + (strips > 1 ? tid % k : tid);
        const int strip = strips > 1 ? tid / k : 0;
        if (j < k && strip < strips && (h == 0 || k > NT)) {
            for (int sl = strip; sl < nslices; sl += strips) {
                const int c = table[size_t(sl) * k + j];
                before[h] += sl < slice ? c : 0;
                total[h] += c;
            }
        }
    }

    for (int q = tid; q < (NWV + 2) * k; q += NT) wh[q] = 0;      // wh, tot and bef are contiguous
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 4; ++c)
        if (key[c] < k) atomicAdd(&wh[wave * k + key[c]], 1);
#pragma unroll
    for (int h = 0; h < GPT; ++h) {
        const int j = h * NT + (strips > 1 ? tid % k : tid);
        const int strip = strips > 1 ? tid / k : 0;
        if (j < k && strip < strips && (h == 0 || k > NT)) {
            atomicAdd(&tot[j], total[h]);
            atomicAdd(&bef[j], before[h]);
        }
    }
    __syncthreads();
    for (int j = tid; j < k; j += NT) {
        int run = bef[j];
#pragma unroll
        for (int w = 0; w < NWV; ++w) {
            const int c = wh[w * k + j];
            wh[w * k + j] = run;
            run += c;
        }
    }
    __syncthreads();

    // exclusive scan of tot[] over the generators, NT at a time
    int carry = 0;
    for (int base = 0; base < k; base += NT) {
        const int j = base + tid;
        const int x = j < k ? tot[j] : 0;
        int incl = x;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int y = __shfl_up(incl, o);
            if (lane >= o) incl += y;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        int wpre = 0, all = 0;
#pragma unroll
        for (int w = 0; w < NWV; ++w) {
            const int v = wsum[w];
            wpre += w < wave ? v : 0;
            all += v;
        }
        const int start = carry + wpre + incl - x;
        if (j < k) {
            tot[j] = start;
            bef[j] = x;                         // bef is free by now: keep the generator's row count for the tail below
        }
        carry += all;
        __syncthreads();
    }
    const int L = carry;                        // the list's length is known now
    if (slice == 0) {                           // chunk size, pieces per generator
        const int P = piece_rows_for(L, wg_cols, p_fixed);
        for (int j = tid; j < k; j += NT) {
            const int start = tot[j], x = bef[j];
            sbase[j] = start / P + j;
            snum[j] = x > 0 ? (start + x - 1) / P - start / P + 1 : 0;
        }
        if (tid == 0) { hdr[0] = L; hdr[1] = P; }
    }

    const int nbits = 32 - __clz(k);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const bool live = key[c] < k;
        const int kc = live ? key[c] : 0;
        const int pos = tot[kc] + stable_slot(&wh[wave * k + kc], live, key[c], nbits);
        if (live) {
            list[pos] = list_entry(i0 + 64 * c, al[c], key[c]);
            if (pos == L - 1) pad_list(list, L, i0 + 64 * c, key[c]);
        }
    }
}

// The same counting sort for batches of at most 4096 Q rows (Q = 1, 2, 4: b <= 16384) in ONE workgroup of 16 waves
// and one kernel: the whole histogram is the workgroup's own, so nothing passes through memory between the two
// phases and one dispatch latency is saved (the small shapes are bound by those).  Wave w owns the rows
// [256 Q w, 256 Q (w + 1)).
template <int Q>
__global__ __launch_bounds__(1024) void k_sort_one(const int32_t* __restrict__ f, const float* __restrict__ alpha, int b, int k,
                                                   int wg_cols, int p_fixed, u32x4_t* __restrict__ list,
                                                   int32_t* __restrict__ sbase, int32_t* __restrict__ snum,
                                                   int32_t* __restrict__ hdr) {
    constexpr int NT = 1024, NWV = 16;
    extern __shared__ int lds[];
    int* wh = lds;                 // [NWV][k] per-wave counts, later per-wave next free position inside the generator's list
    int* tot = lds + NWV * k;      // [k]      rows per generator, later start of the generator's list
    int* cnt = tot + k;            // [k]      rows per generator
    __shared__ int wsum[NWV];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int r0 = wave * (256 * Q);

    int key[Q][4];
    float al[Q][4];
#pragma unroll
    for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int c = 0; c < 4; ++c) key[q][c] = load_key(f, alpha, r0 + (4 * q + c) * 64 + lane, b, k, al[q][c]);      // slot 4 q + c
    for (int q = tid; q < (NWV + 2) * k; q += NT) wh[q] = 0;      // wh, tot and cnt are contiguous
    __syncthreads();
#pragma unroll
    for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (key[q][c] < k) atomicAdd(&wh[wave * k + key[q][c]], 1);
    __syncthreads();
    for (int j = tid; j < k; j += NT) {
        int run = 0;
#pragma unroll
        for (int w = 0; w < NWV; ++w) {
            const int c = wh[w * k + j];
            wh[w * k + j] = run;
            run += c;
        }
        tot[j] = run;
    }
    __syncthreads();

    // exclusive scan of tot[] over the generators, NT at a time
    int carry = 0;
    for (int base = 0; base < k; base += NT) {
        const int j = base + tid;
        const int x = j < k ? tot[j] : 0;
        int incl = x;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int y = __shfl_up(incl, o);
            if (lane >= o) incl += y;
        }
        if (lane == 63) wsum[wave] = incl;
        __syncthreads();
        int wpre = 0, all = 0;
#pragma unroll
        for (int w = 0; w < NWV; ++w) {
            const int v = wsum[w];
            wpre += w < wave ? v : 0;
            all += v;
        }
        const int start = carry + wpre + incl - x;
        if (j < k) {
            tot[j] = start;
            cnt[j] = x;
        }
        carry += all;
        __syncthreads();
    }
    const int L = carry;
    const int P = piece_rows_for(L, wg_cols, p_fixed);
    for (int j = tid; j < k; j += NT) {
        const int start = tot[j], x = cnt[j];
        sbase[j] = start / P + j;
        snum[j] = x > 0 ? (start + x - 1) / P - start / P + 1 : 0;
    }
    if (tid == 0) { hdr[0] = L; hdr[1] = P; }

    const int nbits = 32 - __clz(k);
#pragma unroll
    for (int q = 0; q < Q; ++q) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int row = r0 + (4 * q + c) * 64 + lane;
            const bool live = key[q][c] < k;
            const int kc = live ? key[q][c] : 0;
            const int pos = tot[kc] + stable_slot(&wh[wave * k + kc], live, key[q][c], nbits);
            if (live) {
                list[pos] = list_entry(row, al[q][c], key[q][c]);
                if (pos == L - 1) pad_list(list, L, row, key[q][c]);
            }
        }
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
    // dY is read exactly once: non-temporal loads keep the stream from evicting what is reused (the sorted lists,
    // the partial rows, X and C of the next compression) from L2 and the Infinity Cache
    __device__ __forceinline__ void load(const u32x4_t* __restrict__ rowp, int ch, int) { v = __builtin_nontemporal_load(&rowp[ch]); }
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
    __device__ __forceinline__ void load(const u32x4_t* __restrict__ rowp, int ch, int mch) {
        v0 = __builtin_nontemporal_load(&rowp[ch]);
        v1 = __builtin_nontemporal_load(&rowp[min(ch + 1, mch - 1)]);
    }
    __device__ __forceinline__ void fma(float a, float (&acc)[8]) const {
        acc[0] = fmaf(a, __uint_as_float(v0.x), acc[0]); acc[1] = fmaf(a, __uint_as_float(v0.y), acc[1]);
        acc[2] = fmaf(a, __uint_as_float(v0.z), acc[2]); acc[3] = fmaf(a, __uint_as_float(v0.w), acc[3]);
        acc[4] = fmaf(a, __uint_as_float(v1.x), acc[4]); acc[5] = fmaf(a, __uint_as_float(v1.y), acc[5]);
        acc[6] = fmaf(a, __uint_as_float(v1.z), acc[6]); acc[7] = fmaf(a, __uint_as_float(v1.w), acc[7]);
    }
    static __device__ __forceinline__ int chunk_of(int grp, int lane, int mch) { return min(2 * (grp * 64 + lane), mch - 1); }
};

// Workgroup = 4 waves that share a chunk of the list and sit side by side along the row: wave w covers W
// consecutive 512-column groups, so the workgroup reads 4*W KiB of every row at (nearly) the same time.
template <typename TR, int W>
__global__ __launch_bounds__(256) void k_contract(const u32x4_t* __restrict__ dY, const u32x4_t* __restrict__ list,
                                                  const int32_t* __restrict__ hdr, int mch, int m, int wgcols,
                                                  float* __restrict__ partial) {
    const int chunk = blockIdx.x / wgcols, wc = blockIdx.x % wgcols;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int grp0 = (wc * 4 + wave) * W;
    if (grp0 * 512 >= m) return;                           // this wave has no columns (uniform per wave)
    const int L = __builtin_amdgcn_readfirstlane(hdr[0]), P = __builtin_amdgcn_readfirstlane(hdr[1]);
    const int s0 = chunk * P;
    if (s0 >= L) return;                                   // the list ends before this chunk (uniform per workgroup)
    const int s1 = min(L, s0 + P);
    int ch[W];
#pragma unroll
    for (int w = 0; w < W; ++w) ch[w] = RowLoad<TR>::chunk_of(grp0 + w, lane, mch);

    float acc[W][8];
#pragma unroll
    for (int w = 0; w < W; ++w)
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[w][q] = 0.f;
    int cur = __builtin_amdgcn_readfirstlane(int(list[s0].z));

    // A piece is stored when its generator ends.  Stores in the middle of the stream are expensive here: the one counter
    // that orders a wave's memory operations makes every later wait for loads wait for the older stores as well, and a
    // store takes long to be acknowledged while HBM is busy reading.  So the sums of the generators that end inside the
    // chunk wait in this wave's part of the LDS (up to kHeld of them; LDS traffic has a counter of its own) and go out
    // together when the chunk is done; only a chunk with more generators than that stores in mid-stream.
    constexpr int kHeld = W == 3 ? 6 : 8;                  // 144, 128 or 64 KiB of LDS for the workgroup (one per compute unit)
    __shared__ float4 lds_piece[4][kHeld][W][2][64];       // [wave][slot][column group][half][lane]
    __shared__ int lds_key[4][kHeld];
    int nheld = 0;                                         // wave-uniform
    auto store_piece = [&](const float (&v)[W][8], int key) {
#pragma unroll
        for (int w = 0; w < W; ++w) {
            const int col = (grp0 + w) * 512 + lane * 8;
            if (col < m) {
                float4* dst = reinterpret_cast<float4*>(partial + size_t(chunk + key) * m + col);
                dst[0] = make_float4(v[w][0], v[w][1], v[w][2], v[w][3]);
                if (col + 4 < m) dst[1] = make_float4(v[w][4], v[w][5], v[w][6], v[w][7]);
            }
        }
    };
    auto drain = [&]() {                                   // the held pieces go out, oldest first
        wave_lds_sync();
        for (int h = 0; h < nheld; ++h) {
            const int key = __builtin_amdgcn_readfirstlane(lds_key[wave][h]);
            float v[W][8];
#pragma unroll
            for (int w = 0; w < W; ++w) {
                const float4 lo = lds_piece[wave][h][w][0][lane], hi = lds_piece[wave][h][w][1][lane];
                v[w][0] = lo.x; v[w][1] = lo.y; v[w][2] = lo.z; v[w][3] = lo.w;
                v[w][4] = hi.x; v[w][5] = hi.y; v[w][6] = hi.z; v[w][7] = hi.w;
            }
            store_piece(v, key);
        }
        wave_lds_sync();
        nheld = 0;
    };
    auto flush = [&](int key) {                            // generator `key` ends inside the chunk
        if (nheld == kHeld) drain();
#pragma unroll
        for (int w = 0; w < W; ++w) {
            lds_piece[wave][nheld][w][0][lane] = make_float4(acc[w][0], acc[w][1], acc[w][2], acc[w][3]);
            lds_piece[wave][nheld][w][1][lane] = make_float4(acc[w][4], acc[w][5], acc[w][6], acc[w][7]);
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[w][q] = 0.f;
        }
        if (lane == 0) lds_key[wave][nheld] = key;
        ++nheld;
    };

    // Rows are fetched in groups of U, two groups ahead of the one being summed.  Every step of the loop issues
    // exactly the same number of loads whatever path it takes (positions past the end of the chunk are clamped
    // onto its last group, which is in cache by then), so the wait before a group's sums only has to cover that
    // group and the two younger ones stay in flight.  The sorted list is padded to a multiple of 16 entries
    // (weight 0, last key, a valid row), so a group never needs a guard.
    constexpr int U = (RowLoad<TR>::kGroup / W) < 2 ? 2 : (RowLoad<TR>::kGroup / W);
    static_assert(16 % (2 * U) == 0, "a chunk must be a whole number of group pairs");
    const int last = (s1 + 2 * U - 1) / (2 * U) * (2 * U) - U;      // start of the chunk's last group
    // list entries (row number, weight, generator: wave-uniform, so they travel through scalar registers)
    auto entries_of = [&](int (&row)[U], float (&a)[U], int (&key)[U], int s) {
        s = min(s, last);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const u32x4_t e = list[s + u];
            row[u] = __builtin_amdgcn_readfirstlane(int(e.x));
            a[u] = __uint_as_float(__builtin_amdgcn_readfirstlane(e.y));
            key[u] = __builtin_amdgcn_readfirstlane(int(e.z));
        }
    };
    auto issue = [&](RowLoad<TR> (&v)[U][W], const int (&row)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int w = 0; w < W; ++w) v[u][w].load(dY + size_t(row[u]) * mch, ch[w], mch);
    };
    auto consume = [&](const RowLoad<TR> (&v)[U][W], const float (&a)[U], const int (&key)[U]) {
        if (key[0] == cur && key[U - 1] == cur) {          // the list is sorted: the whole group belongs to `cur`
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int w = 0; w < W; ++w) v[u][w].fma(a[u], acc[w]);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (key[u] != cur) { flush(cur); cur = key[u]; }
#pragma unroll
                for (int w = 0; w < W; ++w) v[u][w].fma(a[u], acc[w]);
            }
        }
    };
    // a: group being summed / next to be issued into the same registers; the entries of a group are fetched when the
    // previous group in the same registers is issued, one step before they are needed
    RowLoad<TR> va[U][W], vb[U][W];
    float aa[U], ab[U], na[U], nb[U];
    int ka[U], kb[U], ra[U], rb[U], nka[U], nkb[U], nra[U], nrb[U];
    entries_of(ra, aa, ka, s0);
    entries_of(rb, ab, kb, s0 + U);
    issue(va, ra);
    issue(vb, rb);
    entries_of(nra, na, nka, s0 + 2 * U);
    entries_of(nrb, nb, nkb, s0 + 3 * U);
    for (int s = s0; s < s1; s += 2 * U) {
        consume(va, aa, ka);
        issue(va, nra);
#pragma unroll
        for (int u = 0; u < U; ++u) { aa[u] = na[u]; ka[u] = nka[u]; }
        entries_of(nra, na, nka, s + 4 * U);
        consume(vb, ab, kb);
        issue(vb, nrb);
#pragma unroll
        for (int u = 0; u < U; ++u) { ab[u] = nb[u]; kb[u] = nkb[u]; }
        entries_of(nrb, nb, nkb, s + 5 * U);
    }
    drain();
    store_piece(acc, cur);
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
// rows padded with zeros to KP generators (whole stages of k_ctb: a multiple of 32 for bf16, 16 for fp32).  A workgroup transposes a tile of 64 columns x 16
// generators through LDS: reads run along the columns (coalesced), writes are whole 16-byte chunks.
template <typename TR> struct PrepIo;
template <> struct PrepIo<Bf16> {
    static constexpr int kChunksPer16 = 2;       // 16 generators = 2 chunks of 8 bf16
    static __device__ __forceinline__ float load_c(const void* C, size_t idx) {
        return __uint_as_float(uint32_t(static_cast<const uint16_t*>(C)[idx]) << 16);
    }
    static __device__ __forceinline__ u32x4_t pack(const float* v) {     // 8 values
        return u32x4_t{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
    }
};
template <> struct PrepIo<F32> {
    static constexpr int kChunksPer16 = 4;       // 16 generators = 4 chunks of 4 fp32
    static __device__ __forceinline__ float load_c(const void* C, size_t idx) { return static_cast<const float*>(C)[idx]; }
    static __device__ __forceinline__ u32x4_t pack(const float* v) {     // 4 values
        return u32x4_t{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
    }
};

template <typename TR>
__global__ __launch_bounds__(256) void k_prep(const void* __restrict__ C, const float* __restrict__ partial,
                                              const int32_t* __restrict__ sbase, const int32_t* __restrict__ snum, int n, int m,
                                              int k, int KC, int blocks_m, const int32_t* __restrict__ eta, int b,
                                              u32x4_t* __restrict__ Ct, u32x4_t* __restrict__ Bt) {
    __shared__ float tile[64][17];
    // normalisation factor of Sec. 3.2: beta = b / (b - eta) with eta rows dropped by the neighbourhood condition
    // (1 without a tolerance; 0 if every row was dropped).  It scales Btilde, hence dW.
    float beta = 1.f;
    if (eta) {
        const int dropped = *eta;
        beta = dropped < b ? float(double(b) / double(b - dropped)) : 0.f;
    }
    const int tid = threadIdx.x;
    const int j0 = blockIdx.y * 16;
    const bool is_b = int(blockIdx.x) < blocks_m;
    const int x0 = (is_b ? blockIdx.x : blockIdx.x - blocks_m) * 64;      // first column (of dY) or hidden index
    const int extent = is_b ? m : n;
    // thread t fills (column t % 64, generator t / 64 + 4 i), i = 0..3: the generator is the same for a whole wave
    const int xx = tid & 63, x = x0 + xx;
    if (is_b) {
        // The four sums of a thread advance together, four or eight pieces each per round, so that a round costs one
        // memory latency for 16 or 32 loads (the number of pieces per generator varies; the loop runs to the longest of the four).
        // Slots past a generator's last piece re-read a valid address and count as 0.
        const int xs = min(x, m - 1);
        int base[4], np[4], npmax = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = j0 + (tid >> 6) + 4 * i;
            const bool ok = j < k && x < m;
            base[i] = ok ? sbase[j] : 0;
            np[i] = ok ? snum[j] : 0;
            npmax = max(npmax, np[i]);
        }
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        auto rounds = [&](auto pieces_per_round) {
            constexpr int R = decltype(pieces_per_round)::value;
            for (int t = 0; t < npmax; t += R) {
                float p[4][R];
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int q = 0; q < R; ++q) p[i][q] = partial[size_t(base[i] + max(0, min(t + q, np[i] - 1))) * m + xs];
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int q = 0; q < R; ++q) v[i] += (t + q < np[i]) ? p[i][q] : 0.f;
            }
        };
        // long lists of pieces (few generators, small batches) are bound by the number of rounds; short ones by the
        // loads themselves, of which the wider round issues more than needed
        if (npmax > 4) rounds(std::integral_constant<int, 8>{});
        else rounds(std::integral_constant<int, 4>{});
#pragma unroll
        for (int i = 0; i < 4; ++i) tile[xx][(tid >> 6) + 4 * i] = v[i] * beta;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int jj = (tid >> 6) + 4 * i, j = j0 + jj;
            tile[xx][jj] = (j < k && x < n) ? PrepIo<TR>::load_c(C, size_t(j) * n + x) : 0.f;
        }
    }
    __syncthreads();
    constexpr int CP = PrepIo<TR>::kChunksPer16;
    if (tid < 64 * CP) {
        const int xx = tid & 63, part = tid >> 6;
        const int x = x0 + xx;
        if (x < extent) {
            u32x4_t out = PrepIo<TR>::pack(&tile[xx][part * TR::kPerChunk]);
            u32x4_t* dst = is_b ? Bt : Ct;
            dst[size_t(x) * KC + blockIdx.y * CP + part] = out;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// k_ctb: dW (n x m) = C^T (n x k) * Btilde (k x m).  Both operands come from k_prep with the generator index
// contiguous (Ct[l][j], Bt[c][j]).  Workgroup tile 128 x 128, 4 waves of 64 x 64; the generator index is walked in
// stages of BK = 4 chunks per row (32 bf16 / 16 fp32: 40 KiB of LDS per workgroup, so three workgroups share a CU;
// eight-chunk stages with two workgroups per CU measured the same at k = 1024 and slower at k = 256), staged through
// LDS with coalesced loads that are issued two stages ahead, double buffered in LDS, one barrier per stage.  LDS rows
// are BK+1 chunks apart, which makes the 16-byte reads of a fragment (32 rows, one chunk column) free of bank
// conflicts.  MFMA step u of a stage takes chunk 2u+g from lane group g, for both operands alike.
//
// Tile order: workgroups are handed to the 8 XCDs round-robin, and every XCD has its own L2.  Workgroup number
// bid therefore takes tile (bid % 8) * ceil(T/8) + bid / 8 of an order that walks the output in strips 8 tiles
// wide, row by row: the 64 tiles an XCD works on at one time form an 8 x 8 block that shares 8 + 8 operand tiles.
//
// The two operands enter alike, so the m x n orientation of the result (the layout of a weight stored as
// outputs x inputs) is the same kernel with the operands exchanged.  OUT16 writes the result rounded to bf16
// (round to nearest even): neighbouring lanes hold neighbouring columns, so each pair of lanes exchanges two of its
// four rows and every lane stores two packed pairs instead of four single values.
template <typename TR, int BK, bool OUT16>
__global__ __launch_bounds__(256) void k_ctb(const u32x4_t* __restrict__ Ct, const u32x4_t* __restrict__ Bt, int n, int m, int KC,
                                             int tiles_n, int tiles_m, int per_xcd, void* __restrict__ dWv) {
    constexpr int RS = BK + 1, TILE = 128 * RS;
    constexpr int SUBS = 256 / BK;               // rows staged per pass of the workgroup
    constexpr int NI = 128 / SUBS;               // passes per operand tile
    __shared__ u32x4_t lds[2][2 * TILE];         // [buffer][128 rows of Ct | 128 rows of Bt]
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 31, g = lane >> 5;
    const int wy = wave >> 1, wx = wave & 1;

    const int L = int(blockIdx.x % 8) * per_xcd + int(blockIdx.x / 8);
    if (L >= tiles_n * tiles_m) return;          // uniform for the workgroup
    int tl, tc;
    {
        const int full = tiles_m / 8, rem = tiles_m % 8, per_strip = tiles_n * 8;
        if (L < full * per_strip) { const int q = L % per_strip; tl = q / 8; tc = (L / per_strip) * 8 + q % 8; }
        else { const int q = L - full * per_strip; tl = q / rem; tc = full * 8 + q % rem; }
    }
    const int l0 = tl * 128, c0 = tc * 128;

    // staging: thread t moves chunk t%BK of rows t/BK + SUBS*i (i = 0..NI-1) of both operand tiles
    const int sub = tid / BK, chunk = tid % BK;
    const u32x4_t* src[2 * NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        src[i] = Ct + size_t(min(l0 + sub + SUBS * i, n - 1)) * KC;
        src[NI + i] = Bt + size_t(min(c0 + sub + SUBS * i, m - 1)) * KC;
    }
    // Two stages travel in registers (stage s in slot s % 2), so that a load has two stages of MFMAs to come back.
    // Rows hold a whole number of stages (k_prep pads with zero generators), so nothing is masked: a mask on the
    // loaded value makes the compiler wait for the load right where it is issued.  Stages past the last one re-read
    // the last one and are never stored.
    const int nst = KC / BK;
    u32x4_t reg[2][2 * NI];
    auto gload = [&](int stage, int slot) {
        const int c = min(stage, nst - 1) * BK + chunk;
#pragma unroll
        for (int i = 0; i < 2 * NI; ++i) reg[slot][i] = src[i][c];
    };
    auto sstore = [&](int buf, int slot) {
#pragma unroll
        for (int i = 0; i < 2 * NI; ++i) lds[buf][(i < NI ? 0 : TILE) + (sub + SUBS * (i % NI)) * RS + chunk] = reg[slot][i];
    };

    f32x16_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int bq = 0; bq < 2; ++bq)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][bq][i] = 0.f;

    gload(0, 0);
    gload(1, 1);
    sstore(0, 0);
    gload(2, 0);
    __syncthreads();
    for (int st = 0; st < nst; st += 2) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {                  // stage st + h: LDS buffer h, register slot h
            const int cur = st + h;
            if (cur < nst) {                           // uniform; false only for the second half of an odd last pair
                const u32x4_t* A = lds[h] + (wy * 64 + r) * RS + g;
                const u32x4_t* B = lds[h] + TILE + (wx * 64 + r) * RS + g;
                u32x4_t a[BK / 2][2], bq[BK / 2][2];
#pragma unroll
                for (int u = 0; u < BK / 2; ++u)
#pragma unroll
                    for (int q = 0; q < 2; ++q) { a[u][q] = A[32 * q * RS + 2 * u]; bq[u][q] = B[32 * q * RS + 2 * u]; }
#pragma unroll
                for (int u = 0; u < BK / 2; ++u)
#pragma unroll
                    for (int fa = 0; fa < 2; ++fa)
#pragma unroll
                        for (int fb = 0; fb < 2; ++fb) TR::mma(a[u][fa], bq[u][fb], acc[fa][fb]);
            }
            if (cur + 1 < nst) sstore(h ^ 1, h ^ 1);
            gload(cur + 3, h ^ 1);                     // the slot is free again
            __syncthreads();
        }
    }

    // D layout of the 32x32 MFMA: register i of lane (r,g) is row 8*(i/4)+4*g+(i%4), column r: one store
    // instruction writes two full 128-byte row segments.  The stores are non-temporal: dW is not read again by this
    // library, and as ordinary stores its dirty lines are written back later, in the middle of the next kernels'
    // streams (measured: 25 % slower k_contract and k_score at the 7B-shaped layer).
    const int lw = l0 + wy * 64, cw = c0 + wx * 64;
    const bool inside = l0 + 128 <= n && c0 + 128 <= m;      // uniform: a tile away from the edges stores unguarded
    if constexpr (!OUT16) {
        float* __restrict__ dW = static_cast<float*>(dWv);
        if (inside) {
            float* __restrict__ base = dW + size_t(lw + 4 * g) * m + cw + r;
#pragma unroll
            for (int fa = 0; fa < 2; ++fa)
#pragma unroll
                for (int fb = 0; fb < 2; ++fb)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        __builtin_nontemporal_store(acc[fa][fb][i], base + size_t(32 * fa + 8 * (i >> 2) + (i & 3)) * m + 32 * fb);
        } else {
#pragma unroll
            for (int fa = 0; fa < 2; ++fa)
#pragma unroll
                for (int fb = 0; fb < 2; ++fb) {
                    const int c = cw + 32 * fb + r;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int l = lw + 32 * fa + 8 * (i >> 2) + 4 * g + (i & 3);
                        if (l < n && c < m) __builtin_nontemporal_store(acc[fa][fb][i], &dW[size_t(l) * m + c]);
                    }
                }
        }
    } else {
        // even lane: keeps rows +0,+1 of each group of four and gets its neighbour's values of those rows (the column
        // to its right); odd lane: keeps rows +2,+3 and gets the column to its left.  m is even, so a pair never
        // straddles the edge.
        uint32_t* __restrict__ dW = static_cast<uint32_t*>(dWv);
        const bool odd = r & 1;
#pragma unroll
        for (int fa = 0; fa < 2; ++fa)
#pragma unroll
            for (int fb = 0; fb < 2; ++fb) {
                const int c = cw + 32 * fb + (r & ~1);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float v0 = acc[fa][fb][4 * q], v1 = acc[fa][fb][4 * q + 1], v2 = acc[fa][fb][4 * q + 2],
                                v3 = acc[fa][fb][4 * q + 3];
                    const float got0 = __shfl_xor(odd ? v0 : v2, 1), got1 = __shfl_xor(odd ? v1 : v3, 1);
                    const uint32_t p0 = odd ? pack_bf16(got0, v2) : pack_bf16(v0, got0);
                    const uint32_t p1 = odd ? pack_bf16(got1, v3) : pack_bf16(v1, got1);
                    const int l = lw + 32 * fa + 8 * q + 4 * g + (odd ? 2 : 0);
                    if (c < m) {
                        if (l < n) __builtin_nontemporal_store(p0, &dW[(size_t(l) * m + c) >> 1]);
                        if (l + 1 < n) __builtin_nontemporal_store(p1, &dW[(size_t(l + 1) * m + c) >> 1]);
                    }
                }
            }
    }
}

// k_prep_rows: the operands of k_ctb_big, which takes them as they are stored (generator index across rows):
//   Bp[j][:] = beta * (sum of generator j's partial rows), rounded once to bf16;   Cp[j][:] = C[j][:];
// both with zero rows from k up to a whole number of 32-generator stages.  One thread per 16-byte chunk of a row.
__global__ __launch_bounds__(256) void k_prep_rows(const u32x4_t* __restrict__ C, const float* __restrict__ partial,
                                                   const int32_t* __restrict__ sbase, const int32_t* __restrict__ snum, int nch,
                                                   int mch, int k, const int32_t* __restrict__ eta, int b,
                                                   u32x4_t* __restrict__ Cp, u32x4_t* __restrict__ Bp) {
    const int j = blockIdx.y;
    const int x = blockIdx.x * 256 + threadIdx.x;               // chunk of the row: first those of Bp, then those of Cp
    if (x < mch) {
        u32x4_t out = {0u, 0u, 0u, 0u};
        if (j < k) {
            float beta = 1.f;                                   // normalisation factor of Sec. 3.2, as in k_prep
            if (eta) {
                const int dropped = *eta;
                beta = dropped < b ? float(double(b) / double(b - dropped)) : 0.f;
            }
            const int base = sbase[j], np = snum[j];
            float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            const size_t row = size_t(mch) * 2;                 // a partial row in float4
            const float4* src = reinterpret_cast<const float4*>(partial) + size_t(base) * row + size_t(x) * 2;
            for (int q = 0; q < np; ++q) {
                const float4 lo = src[size_t(q) * row], hi = src[size_t(q) * row + 1];
                v[0] += lo.x; v[1] += lo.y; v[2] += lo.z; v[3] += lo.w;
                v[4] += hi.x; v[5] += hi.y; v[6] += hi.z; v[7] += hi.w;
            }
            out = u32x4_t{pack_bf16(v[0] * beta, v[1] * beta), pack_bf16(v[2] * beta, v[3] * beta),
                          pack_bf16(v[4] * beta, v[5] * beta), pack_bf16(v[6] * beta, v[7] * beta)};
        }
        Bp[size_t(j) * mch + x] = out;
    } else if (x - mch < nch) {
        const int c = x - mch;
        Cp[size_t(j) * nch + c] = j < k ? C[size_t(j) * nch + c] : u32x4_t{0u, 0u, 0u, 0u};
    }
}

// k_ctb_big: the same product for the shapes where the matrix cores are the limit (many generators, large weight
// gradient; bf16 operands): 256 x 256 tiles on the main loop of pamm_tile256.h, with both operands as they are stored
// (k' x n and k' x m, generator index across rows: the transposing LDS reads of gfx950 deliver the MFMA operands, so
// nothing is transposed through memory); k' is a whole number of 32-generator stages (k_prep_rows pads with zero
// rows).  Tile order, store layout and the bf16 packing are those of k_ctb, over 4 x 4 accumulator fragments per wave.
template <bool OUT16, int FQ>
__global__ __launch_bounds__(256, FQ == 2 ? 2 : 1) void k_ctb_big(const u32x4_t* __restrict__ Rp, const u32x4_t* __restrict__ Qp, int n, int m,
                                                                  int kpad, int tiles_n, int tiles_m, int per_xcd, void* __restrict__ dWv) {
    constexpr int NB = FQ == 2 ? 3 : 4;                    // stage buffers: what fits the LDS with 2 / 1 workgroups per CU
    __shared__ u32x4_t lds[TileLds<NB, FQ>::kChunks];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 31, g = lane >> 5;
    const int wy = wave >> 1, wx = wave & 1;
    const int L = int(blockIdx.x % 8) * per_xcd + int(blockIdx.x / 8);
    if (L >= tiles_n * tiles_m) return;          // uniform for the workgroup
    int tl, tc;
    {
        const int full = tiles_m / 8, rem = tiles_m % 8, per_strip = tiles_n * 8;
        if (L < full * per_strip) { const int q = L % per_strip; tl = q / 8; tc = (L / per_strip) * 8 + q % 8; }
        else { const int q = L - full * per_strip; tl = q / rem; tc = full * 8 + q % rem; }
    }
    const int l0 = tl * 256, c0 = tc * (64 * FQ);
    f32x16_t acc[4][FQ];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int q = 0; q < FQ; ++q)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][q][i] = 0.f;
    const TileSource<FQ> src = tile_source<FQ>(Rp, l0, n, size_t(n / 8), Qp, c0, m, size_t(m / 8));
    tile_mainloop<NB, FQ>(lds, src, kpad / 32, acc);

    const int lw = l0 + wy * 128, cw = c0 + wx * (32 * FQ);
    const bool inside = l0 + 256 <= n && c0 + 64 * FQ <= m;      // uniform: a tile away from the edges stores unguarded
    if constexpr (!OUT16) {
        float* __restrict__ dW = static_cast<float*>(dWv);
#pragma unroll
        for (int fa = 0; fa < 4; ++fa)
#pragma unroll
            for (int fb = 0; fb < FQ; ++fb) {
                const int c = cw + 32 * fb + r;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int l = lw + 32 * fa + 8 * (i >> 2) + 4 * g + (i & 3);
                    if (inside || (l < n && c < m)) __builtin_nontemporal_store(acc[fa][fb][i], &dW[size_t(l) * m + c]);
                }
            }
    } else {
        uint32_t* __restrict__ dW = static_cast<uint32_t*>(dWv);
        const bool odd = r & 1;
#pragma unroll
        for (int fa = 0; fa < 4; ++fa)
#pragma unroll
            for (int fb = 0; fb < FQ; ++fb) {
                const int c = cw + 32 * fb + (r & ~1);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float v0 = acc[fa][fb][4 * q], v1 = acc[fa][fb][4 * q + 1], v2 = acc[fa][fb][4 * q + 2],
                                v3 = acc[fa][fb][4 * q + 3];
                    const float got0 = __shfl_xor(odd ? v0 : v2, 1), got1 = __shfl_xor(odd ? v1 : v3, 1);
                    const uint32_t p0 = odd ? pack_bf16(got0, v2) : pack_bf16(v0, got0);
                    const uint32_t p1 = odd ? pack_bf16(got1, v3) : pack_bf16(v1, got1);
                    const int l = lw + 32 * fa + 8 * q + 4 * g + (odd ? 2 : 0);
                    if (c < m) {
                        if (l < n) __builtin_nontemporal_store(p0, &dW[(size_t(l) * m + c) >> 1]);
                        if (l + 1 < n) __builtin_nontemporal_store(p1, &dW[(size_t(l + 1) * m + c) >> 1]);
                    }
                }
            }
    }
}

// ------------------------------------------------------------------------------------------------
// The random-projection baseline (Sec. 4.6): G = S^T dY, the analogue of the contraction with every token weighting
// every one of the r sketch columns, so it is a dense product with the tokens as contraction index and runs on the
// matrix cores while dY streams once from HBM.
//
// k_sketch_contract.  One wave per (chunk of tokens, 128 columns of dY): NR x 4 accumulator fragments (NR = ceil(r / 32)).
// The four waves of a workgroup sit side by side along the row but never wait for each other: every wave runs its own
// pipeline through its own part of the LDS, so a load that comes back late from HBM holds up one wave, not four (with a
// workgroup barrier per stage the kernel ran at two thirds of this rate).  The tokens are walked in stages of 16 (one
// MFMA step); a wave's stage is 16 rows x 16 chunks of dY (4 KiB) and 16 rows x 4 NR chunks of S, in a ring of LDS
// buffers filled by loads that go from global memory straight into LDS (pamm_tile256.h describes the technique: a load
// instruction of dY takes four rows of the stage, 256 contiguous bytes of each; chunk c of stage row t is kept at
// c ^ 4 (t % 4)), and both MFMA operands come out of transposing LDS reads: both matrices have the contraction index
// across their rows.  S is tiny next to dY; the lanes of its loads that fall past the end of the tokens or of the
// sketch's columns fetch a chunk of zeros instead, which also makes the rows of dY past the end (clamped onto the last
// row) count for nothing.  Workgroup 0 leaves the table of pieces for the kernels of the small product.
// Output: one partial row of G per sketch column and chunk, partial[(j chunks + chunk) m + c], which those kernels
// then sum like the pieces of a generator.
template <int NR>
struct SketchLds {
    static constexpr int kNB = NR == 1 ? 7 : (NR == 2 ? 6 : (NR == 3 ? 5 : 4));      // stage buffers that fit the LDS
    static constexpr int kStageY = 256;                         // chunks: 16 rows x 128 columns of bf16
    static constexpr int kStageS = 64 * NR;                     // 16 rows x 4 NR chunks
    static constexpr int kStage = kStageY + kStageS;            // of one wave
    static_assert(4 * kNB * kStage * 16 <= 152 * 1024, "the stage rings do not fit the LDS of a compute unit");
};

// The wave's walk.  (A function of its own with __restrict__ sources on purpose: that is what lets the compiler keep
// the LDS reads apart from the loads into LDS still in flight; in the kernel's own body it makes every LDS read wait for
// ALL outstanding loads, which empties the pipeline at every stage.  The waits that matter are the counted ones below.)
template <int NR>
__device__ __forceinline__ void sketch_contract_wave(u32x4_t* __restrict__ lds, const u32x4_t* __restrict__ S,
                                                     const u32x4_t* __restrict__ dY, const u32x4_t* __restrict__ zero, int b, int rch,
                                                     int mch, int m, int chunk, int chunks, int t0, int nst, int c0, int r,
                                                     float* __restrict__ partial) {
    typedef SketchLds<NR> L;
    typedef __attribute__((ext_vector_type(4))) short s16x4_t;
    typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
    constexpr int NB = L::kNB, NLW = 4 + NR;                     // NLW: loads per stage
    const int lane = threadIdx.x & 63, rr = lane & 31, g = lane >> 5;

    // this lane's part of the loads of a stage: for dY row and column chunk, for S row and chunk
    const int yrow = lane >> 4;                                  // + 4 i for load i
    const int ycol = min(c0 / 8 + ((lane & 15) ^ ((yrow & 3) << 2)), mch - 1);
    int srow[NR], scol[NR];
#pragma unroll
    for (int i = 0; i < NR; ++i) {
        const int q = 64 * i + lane;                             // chunk of the S stage, row-major with 4 NR chunks per row
        srow[i] = q / (4 * NR);
        scol[i] = (q % (4 * NR) < rch) ? q % (4 * NR) : -1;
    }
    auto issue = [&](int stage, int buf) {
        stage = min(stage, nst - 1);                             // past the end: the last stage once more, into a free buffer
        const int tbase = t0 + 16 * stage;
        u32x4_t* const dst = lds + buf * L::kStage;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int tok = min(tbase + 4 * i + yrow, b - 1);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(dY + size_t(tok) * mch + ycol),
                                             (__attribute__((address_space(3))) void*)(dst + i * 64), 16, 0, 2 /* nt: read once */);
        }
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            const int tok = tbase + srow[i];
            const u32x4_t* src = (scol[i] >= 0 && tok < b) ? S + size_t(tok) * rch + scol[i] : zero;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(dst + L::kStageY + 64 * i), 16, 0, 0);
        }
    };
    // fragment addresses inside a stage buffer in 16-bit elements, for the two transposing reads of a fragment (this
    // lane addresses stage row t, columns col .. col + 3 of a 4 x 16 block)
    int off_y[2], off_s[2], frag_y[4];
    {
        const int G = lane >> 4, p = lane & 15, kk = (p >> 2) & 3;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int t = 8 * (G >> 1) + 4 * h + (p >> 2);       // t % 4 == kk
            const int col = 16 * (G & 1) + 4 * (p & 3);
            off_y[h] = t * 128 + col;
            off_s[h] = L::kStageY * 8 + t * (32 * NR) + col;
        }
#pragma unroll
        for (int f = 0; f < 4; ++f) frag_y[f] = 8 * ((4 * f) ^ (kk << 2));
    }
    auto read_frag = [&](const short* base, int o0, int o1) {
        const u32x2_t lo = __builtin_bit_cast(u32x2_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(base + o0)));
        const u32x2_t hi = __builtin_bit_cast(u32x2_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(base + o1)));
        return u32x4_t{lo.x, lo.y, hi.x, hi.y};
    };
    f32x16_t acc[NR][4];
#pragma unroll
    for (int a = 0; a < NR; ++a)
#pragma unroll
        for (int f = 0; f < 4; ++f)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][f][i] = 0.f;

    // Nothing here crosses waves: a wave's LDS reads follow its own loads (counted wait), and its loads into a buffer
    // follow its own reads of that buffer, whose results the MFMAs of the previous round have consumed.
    for (int d = 0; d < NB - 1; ++d) issue(d, d);
    int cur = 0, load_buf = NB - 1;
    for (int s = 0; s < nst; ++s) {
        wait_vmcnt<NLW * (NB - 2)>();             // stage s has landed (the younger ones stay in flight)
        __builtin_amdgcn_sched_barrier(0);
        const short* base = reinterpret_cast<const short*>(lds + cur * L::kStage);
        u32x4_t fs[NR], fy[4];
#pragma unroll
        for (int a = 0; a < NR; ++a) fs[a] = read_frag(base, off_s[0] + 32 * a, off_s[1] + 32 * a);
#pragma unroll
        for (int f = 0; f < 4; ++f) fy[f] = read_frag(base, off_y[0] + frag_y[f], off_y[1] + frag_y[f]);
#pragma unroll
        for (int a = 0; a < NR; ++a)
#pragma unroll
            for (int f = 0; f < 4; ++f) Bf16::mma(fs[a], fy[f], acc[a][f]);
        __builtin_amdgcn_sched_barrier(0);
        issue(s + NB - 1, load_buf);              // into the buffer read one stage ago
        cur = cur + 1 == NB ? 0 : cur + 1;
        load_buf = load_buf + 1 == NB ? 0 : load_buf + 1;
    }
    wait_vmcnt<0>();

    // register i of acc[a][f]: sketch column 32 a + 8 (i / 4) + 4 g + i % 4, column c0 + 32 f + rr
#pragma unroll
    for (int a = 0; a < NR; ++a)
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            const int c = c0 + 32 * f + rr;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int j = 32 * a + 8 * (i >> 2) + 4 * g + (i & 3);
                if (j < r && c < m) partial[(size_t(j) * chunks + chunk) * m + c] = acc[a][f][i];
            }
        }
}

template <int NR>
__global__ __launch_bounds__(256) void k_sketch_contract(const u32x4_t* __restrict__ S, const u32x4_t* __restrict__ dY,
                                                         u32x4_t* __restrict__ zero, int b, int rch, int mch, int m,
                                                         int col_groups, int chunk_rows, int chunks, int r,
                                                         int32_t* __restrict__ sbase, int32_t* __restrict__ snum,
                                                         float* __restrict__ partial) {
    typedef SketchLds<NR> L;
    __shared__ u32x4_t lds_all[4 * L::kNB * L::kStage];
    const int wave = threadIdx.x >> 6;
    const int chunk = blockIdx.x / col_groups, cg = blockIdx.x % col_groups;
    const int t0 = chunk * chunk_rows, t1 = min(b, t0 + chunk_rows);
    // The chunk of zeros: every workgroup writes the same 16 bytes and reads back only what it wrote itself, so the
    // workgroup barrier is all the ordering it takes (a device-wide fence here cost a fifth of the kernel's time).
    // From workgroup 0, the table of pieces: sketch column j owns the partial rows j chunks .. j chunks + chunks - 1.
    if (threadIdx.x == 0) *zero = u32x4_t{0u, 0u, 0u, 0u};
    if (blockIdx.x == 0 && threadIdx.x < r) { sbase[threadIdx.x] = int(threadIdx.x) * chunks; snum[threadIdx.x] = chunks; }
    __syncthreads();
    const int c0 = cg * 512 + wave * 128;                        // this wave's first column
    if (c0 >= m) return;                                         // this wave has no columns (uniform per wave)
    sketch_contract_wave<NR>(lds_all + wave * (L::kNB * L::kStage), S, dY, zero, b, rch, mch, m, chunk, chunks, t0, (t1 - t0 + 15) / 16,
                             c0, r, partial);
}

// The same for fp32 elements.  The fp32 MFMA takes one element per lane and step, so no transposition is needed: a wave
// covers 64 columns (stage: 16 tokens x 16 chunks of dY, 16 x 8 NR chunks of S), chunk c of stage row t sits at
// c ^ 8 (t % 2) so that the two token rows one step reads fall into different banks, and every MFMA operand is a plain
// 4-byte LDS read.
template <int NR>
struct SketchLdsF32 {
    static constexpr int kNB = NR == 1 ? 6 : (NR == 2 ? 4 : 3);
    static constexpr int kStageY = 256;                         // chunks: 16 rows x 64 columns of fp32
    static constexpr int kStageS = 128 * NR;                    // 16 rows x 8 NR chunks
    static constexpr int kStage = kStageY + kStageS;            // of one wave
    static_assert(4 * kNB * kStage * 16 <= 152 * 1024, "the stage rings do not fit the LDS of a compute unit");
};

template <int NR>
__device__ __forceinline__ void sketch_contract_wave_f32(u32x4_t* __restrict__ lds, const u32x4_t* __restrict__ S,
                                                         const u32x4_t* __restrict__ dY, const u32x4_t* __restrict__ zero, int b,
                                                         int rch, int mch, int m, int chunk, int chunks, int t0, int nst, int c0, int r,
                                                         float* __restrict__ partial) {
    typedef SketchLdsF32<NR> L;
    constexpr int NB = L::kNB, NLW = 4 + 2 * NR;                 // NLW: loads per stage
    const int lane = threadIdx.x & 63, rr = lane & 31, g = lane >> 5;

    const int yrow = lane >> 4;                                  // + 4 i for load i
    const int ycol = min(c0 / 4 + ((lane & 15) ^ ((yrow & 1) << 3)), mch - 1);
    int srow[2 * NR], scol[2 * NR];
#pragma unroll
    for (int i = 0; i < 2 * NR; ++i) {
        const int q = 64 * i + lane;                             // chunk of the S stage, row-major with 8 NR chunks per row
        srow[i] = q / (8 * NR);
        scol[i] = (q % (8 * NR) < rch) ? q % (8 * NR) : -1;
    }
    auto issue = [&](int stage, int buf) {
        stage = min(stage, nst - 1);                             // past the end: the last stage once more, into a free buffer
        const int tbase = t0 + 16 * stage;
        u32x4_t* const dst = lds + buf * L::kStage;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int tok = min(tbase + 4 * i + yrow, b - 1);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(dY + size_t(tok) * mch + ycol),
                                             (__attribute__((address_space(3))) void*)(dst + i * 64), 16, 0, 2 /* nt: read once */);
        }
#pragma unroll
        for (int i = 0; i < 2 * NR; ++i) {
            const int tok = tbase + srow[i];
            const u32x4_t* src = (scol[i] >= 0 && tok < b) ? S + size_t(tok) * rch + scol[i] : zero;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(dst + L::kStageY + 64 * i), 16, 0, 0);
        }
    };
    // float offsets inside a stage buffer: step ks takes tokens 2 ks + g; the swizzle of the dY rows only depends on g
    int off_y[2];
#pragma unroll
    for (int f = 0; f < 2; ++f) off_y[f] = g * 64 + 4 * ((8 * f + (rr >> 2)) ^ (g << 3)) + (rr & 3);
    const int off_s = L::kStageY * 4 + g * (32 * NR) + rr;
    f32x16_t acc[NR][2];
#pragma unroll
    for (int a = 0; a < NR; ++a)
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][f][i] = 0.f;

    for (int d = 0; d < NB - 1; ++d) issue(d, d);
    int cur = 0, load_buf = NB - 1;
    for (int s = 0; s < nst; ++s) {
        wait_vmcnt<NLW * (NB - 2)>();             // stage s has landed (the younger ones stay in flight)
        __builtin_amdgcn_sched_barrier(0);
        const float* base = reinterpret_cast<const float*>(lds + cur * L::kStage);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            float fs[NR], fy[2];
#pragma unroll
            for (int a = 0; a < NR; ++a) fs[a] = base[off_s + ks * (64 * NR) + 32 * a];
#pragma unroll
            for (int f = 0; f < 2; ++f) fy[f] = base[off_y[f] + ks * 128];
#pragma unroll
            for (int a = 0; a < NR; ++a)
#pragma unroll
                for (int f = 0; f < 2; ++f) acc[a][f] = __builtin_amdgcn_mfma_f32_32x32x2f32(fs[a], fy[f], acc[a][f], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        issue(s + NB - 1, load_buf);              // into the buffer read one stage ago
        cur = cur + 1 == NB ? 0 : cur + 1;
        load_buf = load_buf + 1 == NB ? 0 : load_buf + 1;
    }
    wait_vmcnt<0>();

#pragma unroll
    for (int a = 0; a < NR; ++a)
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            const int c = c0 + 32 * f + rr;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int j = 32 * a + 8 * (i >> 2) + 4 * g + (i & 3);
                if (j < r && c < m) partial[(size_t(j) * chunks + chunk) * m + c] = acc[a][f][i];
            }
        }
}

template <int NR>
__global__ __launch_bounds__(256) void k_sketch_contract_f32(const u32x4_t* __restrict__ S, const u32x4_t* __restrict__ dY,
                                                             u32x4_t* __restrict__ zero, int b, int rch, int mch, int m,
                                                             int col_groups, int chunk_rows, int chunks, int r,
                                                             int32_t* __restrict__ sbase, int32_t* __restrict__ snum,
                                                             float* __restrict__ partial) {
    typedef SketchLdsF32<NR> L;
    __shared__ u32x4_t lds_all[4 * L::kNB * L::kStage];
    const int wave = threadIdx.x >> 6;
    const int chunk = blockIdx.x / col_groups, cg = blockIdx.x % col_groups;
    const int t0 = chunk * chunk_rows, t1 = min(b, t0 + chunk_rows);
    if (threadIdx.x == 0) *zero = u32x4_t{0u, 0u, 0u, 0u};       // as in k_sketch_contract
    if (blockIdx.x == 0 && threadIdx.x < r) { sbase[threadIdx.x] = int(threadIdx.x) * chunks; snum[threadIdx.x] = chunks; }
    __syncthreads();
    const int c0 = cg * 256 + wave * 64;                         // this wave's first column
    if (c0 >= m) return;                                         // this wave has no columns (uniform per wave)
    sketch_contract_wave_f32<NR>(lds_all + wave * (L::kNB * L::kStage), S, dY, zero, b, rch, mch, m, chunk, chunks, t0,
                                 (t1 - t0 + 15) / 16, c0, r, partial);
}

// ------------------------------------------------------------------------------------------------ host side

struct GradBuffers {
    int32_t *sbase, *snum, *table, *hdr;
    float* partial;
    u32x4_t *list, *ct, *bt;
};

static GradBuffers carve(const GradPlan& pl, char* ws) {
    GradBuffers g;
    g.list = reinterpret_cast<u32x4_t*>(ws + pl.off_list);
    g.sbase = reinterpret_cast<int32_t*>(ws + pl.off_sbase);
    g.snum = reinterpret_cast<int32_t*>(ws + pl.off_snum);
    g.table = reinterpret_cast<int32_t*>(ws + pl.off_table);
    g.hdr = reinterpret_cast<int32_t*>(ws + pl.off_hdr);
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
        if (k <= kScatterMaxK && b <= pl.sort_one_rows) {
            const size_t lds = size_t(16 + 2) * k * 4;
#define PAMM_LAUNCH_SORT_ONE(QV) \
    hipLaunchKernelGGL(k_sort_one<QV>, dim3(1), dim3(1024), lds, s, f, alpha, b, k, pl.wg_cols, pl.p_fixed, g.list, g.sbase, g.snum, \
                       g.hdr)
            if (b <= 4096) PAMM_LAUNCH_SORT_ONE(1);
            else if (b <= 8192) PAMM_LAUNCH_SORT_ONE(2);
            else PAMM_LAUNCH_SORT_ONE(4);
#undef PAMM_LAUNCH_SORT_ONE
        } else if (k <= kScatterMaxK) {
            const int nslices = int(pl.nslices);
            if (pl.slice_rows == 1024) {
                hipLaunchKernelGGL(k_hist<256>, dim3(nslices), dim3(256), size_t(k) * 4, s, f, alpha, b, k, g.table);
                hipLaunchKernelGGL(k_scatter<256>, dim3(nslices), dim3(256), size_t(4 + 2) * k * 4, s, f, alpha, b, k, pl.wg_cols,
                                   pl.p_fixed, nslices, g.table, g.list, g.sbase, g.snum, g.hdr);
            } else {
                hipLaunchKernelGGL(k_hist<1024>, dim3(nslices), dim3(1024), size_t(k) * 4, s, f, alpha, b, k, g.table);
                hipLaunchKernelGGL(k_scatter<1024>, dim3(nslices), dim3(1024), size_t(16 + 2) * k * 4, s, f, alpha, b, k,
                                   pl.wg_cols, pl.p_fixed, nslices, g.table, g.list, g.sbase, g.snum, g.hdr);
            }
        } else {
#define PAMM_LAUNCH_GROUP(KERNEL) \
    hipLaunchKernelGGL(KERNEL, dim3(k), dim3(1024), 0, s, f, alpha, b, k, pl.wg_cols, pl.p_fixed, g.list, g.sbase, g.snum, g.hdr)
        const int nv = (b + 4095) / 4096;      // int4 loads per lane when 16 waves share the rows
        if (nv <= 1) PAMM_LAUNCH_GROUP(k_group_regs<1>);
        else if (nv <= 2) PAMM_LAUNCH_GROUP(k_group_regs<2>);
        else if (nv <= 4) PAMM_LAUNCH_GROUP(k_group_regs<4>);
        else if (nv <= 8) PAMM_LAUNCH_GROUP(k_group_regs<8>);
        else if (nv <= 16) PAMM_LAUNCH_GROUP(k_group_regs<16>);
        else PAMM_LAUNCH_GROUP(k_group_stream);
#undef PAMM_LAUNCH_GROUP
        }
    }
    const int mch = m / TR::kPerChunk;
    {
        ScopedSpan span(kContract, s);
        const dim3 grid((unsigned)(pl.chunks * pl.wg_cols));
#define PAMM_LAUNCH_CONTRACT(WV) \
    hipLaunchKernelGGL((k_contract<TR, WV>), grid, dim3(256), 0, s, (const u32x4_t*)dY, g.list, g.hdr, mch, m, pl.wg_cols, \
                       g.partial)
        if (pl.wave_groups == 1) PAMM_LAUNCH_CONTRACT(1);
        else if (pl.wave_groups == 2) PAMM_LAUNCH_CONTRACT(2);
        else PAMM_LAUNCH_CONTRACT(3);
#undef PAMM_LAUNCH_CONTRACT
    }
}

template <typename TR>
static void launch_prep_ctb(const GradPlan& pl, const GradBuffers& g, const void* C, int n, int m, int k, const int32_t* eta, int b,
                            void* dW, bool out16, bool m_by_n, hipStream_t s) {
    if (pl.big_tiles) {
        if constexpr (std::is_same<TR, Bf16>::value) {
            const int nch = n / 8, mch = m / 8, kpad = int(pl.kpad);
            {
                ScopedSpan span(kPrep, s);
                hipLaunchKernelGGL(k_prep_rows, dim3((unsigned)((nch + mch + 255) / 256), (unsigned)kpad), dim3(256), 0, s,
                                   (const u32x4_t*)C, g.partial, g.sbase, g.snum, nch, mch, k, eta, b, g.ct, g.bt);
            }
            // rows x cols of the result: n x m (O = A^T B), or m x n with the operands exchanged
            const u32x4_t* rows_op = m_by_n ? g.bt : g.ct;
            const u32x4_t* cols_op = m_by_n ? g.ct : g.bt;
            const int nr = m_by_n ? m : n, nc = m_by_n ? n : m;
            const bool wide = g_plan_override.small_tiles == 2;          // test hook: 256 x 256 tiles, one workgroup per CU
            const int tiles_r = (nr + 255) / 256, tiles_c = wide ? (nc + 255) / 256 : (nc + 127) / 128;
            const int per_xcd = (tiles_r * tiles_c + 7) / 8;
            ScopedSpan span(kCtb, s);
            const dim3 grid((unsigned)(per_xcd * 8));
            auto launch = [&](auto kernel) {
                hipLaunchKernelGGL(kernel, grid, dim3(256), 0, s, rows_op, cols_op, nr, nc, kpad, tiles_r, tiles_c, per_xcd, dW);
            };
            if (wide) { if (out16) launch(k_ctb_big<true, 4>); else launch(k_ctb_big<false, 4>); }
            else      { if (out16) launch(k_ctb_big<true, 2>); else launch(k_ctb_big<false, 2>); }
        }
        return;
    }
    const int KC = int(pl.kpad) / TR::kPerChunk;
    const int blocks_m = (m + 63) / 64, blocks_n = (n + 63) / 64;
    {
        ScopedSpan span(kPrep, s);
        hipLaunchKernelGGL((k_prep<TR>), dim3((unsigned)(blocks_m + blocks_n), (unsigned)(pl.kpad / 16)), dim3(256), 0, s, C,
                           g.partial, g.sbase, g.snum, n, m, k, KC, blocks_m, eta, b, g.ct, g.bt);
    }
    // rows x cols of the result: n x m (O = A^T B), or m x n with the operands exchanged
    const u32x4_t* rows_op = m_by_n ? g.bt : g.ct;
    const u32x4_t* cols_op = m_by_n ? g.ct : g.bt;
    const int nr = m_by_n ? m : n, nc = m_by_n ? n : m;
    const int tiles_r = (nr + 127) / 128, tiles_c = (nc + 127) / 128;
    const int per_xcd = (tiles_r * tiles_c + 7) / 8;
    {
        ScopedSpan span(kCtb, s);
        const dim3 grid((unsigned)(per_xcd * 8));
        if (out16)
            hipLaunchKernelGGL((k_ctb<TR, 4, true>), grid, dim3(256), 0, s, rows_op, cols_op, nr, nc, KC, tiles_r, tiles_c, per_xcd, dW);
        else
            hipLaunchKernelGGL((k_ctb<TR, 4, false>), grid, dim3(256), 0, s, rows_op, cols_op, nr, nc, KC, tiles_r, tiles_c, per_xcd, dW);
    }
}

}  // namespace pamm

using namespace pamm;

extern "C" pamm_status pamm_contract(const int32_t* f, const float* alpha, const void* dY, int64_t b, int64_t k, int64_t m,
                                     pamm_dtype dt, float* Btilde, void* ws, size_t ws_bytes, void* stream) {
    GradPlan pl;
    pamm_status st = check_contract_args(f, alpha, dY, b, k, m, dt, Btilde, ws, ws_bytes, &pl);
    if (st != PAMM_OK) return st;
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

static pamm_status grad_impl(const void* C, const int32_t* f, const float* alpha, const int32_t* eta, const void* dY, int64_t b,
                             int64_t n, int64_t k, int64_t m, pamm_dtype dt, pamm_dtype out_dt, pamm_layout layout, void* dW,
                             void* ws, size_t ws_bytes, void* stream) {
    GradPlan pl;
    pamm_status st = check_grad_args(C, f, alpha, dY, b, n, k, m, dt, out_dt, layout, dW, ws, ws_bytes, &pl);
    if (st != PAMM_OK) return st;
    const bool out16 = out_dt == PAMM_BF16, m_by_n = layout == PAMM_DW_M_BY_N;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    GradBuffers g = carve(pl, (char*)ws);
    if (dt == PAMM_BF16) {
        launch_group_contract<Bf16>(pl, g, f, alpha, dY, int(b), int(k), int(m), s);
        launch_prep_ctb<Bf16>(pl, g, C, int(n), int(m), int(k), eta, int(b), dW, out16, m_by_n, s);
    } else {
        launch_group_contract<F32>(pl, g, f, alpha, dY, int(b), int(k), int(m), s);
        launch_prep_ctb<F32>(pl, g, C, int(n), int(m), int(k), eta, int(b), dW, out16, m_by_n, s);
    }
    return hipGetLastError() == hipSuccess ? PAMM_OK : PAMM_ERR_DEVICE;
}

// ---- pamm_grad_static: pamm_grad for callers that cannot allocate.  The scratch memory that pamm_grad takes from its
// caller (sorted list, per-generator piece ranges, slice histograms, partial rows, the two operands of the product)
// lives in this file-scope device array instead; every GPU the library runs on holds its own copy at its own address
// until the process ends.  The array's name is only a host-side stand-in: the address on the current device is looked
// up once per device with hipGetSymbolAddress and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[PAMM_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static pamm_status static_scratch(void** out) {
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return PAMM_ERR_DEVICE;
    void* p = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (!p) {          // first call on this device (two first calls at once look up the same address twice: harmless)
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PAMM_ERR_DEVICE;
        g_scratch_ptr[device].store(p, std::memory_order_release);
    }
    *out = p;
    return PAMM_OK;
}

extern "C" pamm_status pamm_grad_static(const void* C, const int32_t* f, const float* alpha, const void* dY, int64_t b, int64_t n,
                                        int64_t k, int64_t m, pamm_dtype dt, float* dW, void* stream) {
    // sizes first: a request that does not fit the array is refused before the device is touched
    const size_t need = pamm_grad_workspace(b, n, k, m, dt);
    if (need > size_t(PAMM_STATIC_SCRATCH_BYTES)) return PAMM_ERR_WORKSPACE;
    void* ws = reinterpret_cast<void*>(uintptr_t(256));          // stands in for the array while the arguments are checked
    GradPlan pl;
    pamm_status st = check_grad_args(C, f, alpha, dY, b, n, k, m, dt, PAMM_F32, PAMM_DW_N_BY_M, dW, ws, PAMM_STATIC_SCRATCH_BYTES, &pl);
    if (st != PAMM_OK) return st;
    st = static_scratch(&ws);
    if (st != PAMM_OK) return st;
    // nothing in the scratch layout has to start at zero: every kernel writes what the next one reads
    return grad_impl(C, f, alpha, nullptr, dY, b, n, k, m, dt, PAMM_F32, PAMM_DW_N_BY_M, dW, ws, PAMM_STATIC_SCRATCH_BYTES, stream);
}

extern "C" pamm_status pamm_grad(const void* C, const int32_t* f, const float* alpha, const void* dY, int64_t b, int64_t n,
                                 int64_t k, int64_t m, pamm_dtype dt, float* dW, void* ws, size_t ws_bytes, void* stream) {
    return grad_impl(C, f, alpha, nullptr, dY, b, n, k, m, dt, PAMM_F32, PAMM_DW_N_BY_M, dW, ws, ws_bytes, stream);
}

extern "C" pamm_status pamm_grad_eps(const void* C, const int32_t* f, const float* alpha, const int32_t* eta, const void* dY,
                                     int64_t b, int64_t n, int64_t k, int64_t m, pamm_dtype dt, float* dW, void* ws,
                                     size_t ws_bytes, void* stream) {
    if (!eta || !aligned4(eta)) return PAMM_ERR_INVALID_ARG;
    return grad_impl(C, f, alpha, eta, dY, b, n, k, m, dt, PAMM_F32, PAMM_DW_N_BY_M, dW, ws, ws_bytes, stream);
}

extern "C" pamm_status pamm_grad_out(const void* C, const int32_t* f, const float* alpha, const int32_t* eta, const void* dY,
                                     int64_t b, int64_t n, int64_t k, int64_t m, pamm_dtype dt, pamm_dtype out_dt,
                                     pamm_layout layout, void* dW, void* ws, size_t ws_bytes, void* stream) {
    if (eta && !aligned4(eta)) return PAMM_ERR_INVALID_ARG;
    return grad_impl(C, f, alpha, eta, dY, b, n, k, m, dt, out_dt, layout, dW, ws, ws_bytes, stream);
}

extern "C" pamm_status pamm_sketch_grad(const void* Pt, const void* S, const void* dY, int64_t b, int64_t n, int64_t r, int64_t m,
                                        pamm_dtype dt, float* dW, void* ws, size_t ws_bytes, void* stream) {
    SketchGradPlan pl;
    pamm_status st = check_sketch_grad_args(Pt, S, dY, b, n, r, m, dt, dW, ws, ws_bytes, &pl);
    if (st != PAMM_OK) return st;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    GradBuffers g = carve(pl.g, (char*)ws);
    u32x4_t* zero = reinterpret_cast<u32x4_t*>((char*)ws + pl.off_zero);
    {
        ScopedSpan span(kSketchContract, s);
        const dim3 grid((unsigned)(pl.chunks * pl.col_groups));
        const int per = dt == PAMM_BF16 ? 8 : 4;
#define PAMM_LAUNCH_SKETCH_CONTRACT(KERNEL, NRV)                                                                                 \
    hipLaunchKernelGGL(KERNEL<NRV>, grid, dim3(256), 0, s, (const u32x4_t*)S, (const u32x4_t*)dY, zero, int(b), int(r / per),   \
                       int(m / per), int(m), pl.col_groups, int(pl.chunk_rows), int(pl.chunks), int(r), g.sbase, g.snum, g.partial)
#define PAMM_SKETCH_CONTRACT_NR(KERNEL)                              \
    do {                                                             \
        if (pl.nr == 1) PAMM_LAUNCH_SKETCH_CONTRACT(KERNEL, 1);      \
        else if (pl.nr == 2) PAMM_LAUNCH_SKETCH_CONTRACT(KERNEL, 2); \
        else if (pl.nr == 3) PAMM_LAUNCH_SKETCH_CONTRACT(KERNEL, 3); \
        else PAMM_LAUNCH_SKETCH_CONTRACT(KERNEL, 4);                 \
    } while (0)
        if (dt == PAMM_BF16) PAMM_SKETCH_CONTRACT_NR(k_sketch_contract);
        else PAMM_SKETCH_CONTRACT_NR(k_sketch_contract_f32);
#undef PAMM_SKETCH_CONTRACT_NR
#undef PAMM_LAUNCH_SKETCH_CONTRACT
    }
    if (dt == PAMM_F32) {
        launch_prep_ctb<F32>(pl.g, g, Pt, int(n), int(m), int(r), nullptr, int(b), dW, false, false, s);
        return hipGetLastError() == hipSuccess ? PAMM_OK : PAMM_ERR_DEVICE;
    }
    launch_prep_ctb<Bf16>(pl.g, g, Pt, int(n), int(m), int(r), nullptr, int(b), dW, false, false, s);
    return hipGetLastError() == hipSuccess ? PAMM_OK : PAMM_ERR_DEVICE;
}
