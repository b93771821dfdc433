// Main loop of a 256 x (64 FQ) tile of a product R^T Q of two bf16 matrices stored row-major with the contraction index
// across their rows (R is K x nr and gives the rows of the result, Q is K x nq and gives its columns), for the shapes
// where the matrix cores are the limit.  Used by the small product of ApproxMM, dW = C^T Btilde (contraction over the
// generators): both operands are taken as they are stored.
//
// Workgroup = 4 waves in a 2 x 2 arrangement, each with a 128 x (32 FQ) part of the tile: 4 x FQ MFMA 32x32x16
// accumulators.  FQ = 4: 256 accumulator registers, one wave per SIMD, one workgroup per compute unit.  FQ = 2: 128
// accumulator registers, two workgroups per compute unit, so that one workgroup's stores of its finished tile and the
// fill of its next pipeline run under the other one's MFMAs.
//
// The contraction index is walked in stages of 32 matrix rows (two MFMA steps); the stages sit in a ring of LDS buffers
// filled by loads that go from global memory straight into LDS (no register hop: a wave has no registers to spare next
// to its accumulators, and nothing has to be waited for in the middle of the MFMA stream).  Such a load writes its 64
// lanes' 16 bytes to consecutive LDS addresses, so the layout is chosen through WHICH chunk a lane fetches: a load
// instruction takes whole matrix rows of the tile (2 rows x 32 chunks of R, 64 / (8 FQ) rows x 8 FQ chunks of Q), and
// chunk c of stage row k is kept at position c ^ 4 (k % 4).  The MFMA operands (for one result row / column, 8
// consecutive contraction indices per lane) come out of the transposing LDS read of gfx950, ds_read_b64_tr_b16: within
// 16 lanes, lane 4a+e receives element e of the 8-byte pieces addressed by lanes a, a+4, a+8, a+12 -- lane q addresses
// row q/4, columns 4 (q%4) .. +3 of a 4 x 16 block and every lane ends up with 4 consecutive rows of ONE column; two
// such reads make one operand.  The swizzle puts the four rows that one read touches into four different 64-byte bank
// groups.  Inside an MFMA step the LDS reads of the next step's fragments and the loads of a later stage are issued one
// by one between the MFMAs, and the only wait is the one before the workgroup barrier in the middle of every stage.
#pragma once

#include "pamm_device.h"

namespace pamm {

template <int NB, int FQ>
struct TileLds {
    static_assert(FQ == 2 || FQ == 4, "the tile is 256 x 128 or 256 x 256");
    static constexpr int kStageR = 1024;                              // chunks: 32 rows x 256 columns of bf16
    static constexpr int kStageQ = 256 * FQ;                          // 32 rows x 64 FQ columns
    static constexpr int kStage = kStageR + kStageQ;
    static constexpr int kChunks = NB * kStage;
    static_assert(NB >= 3, "one stage consumed, one awaited, at least one in flight");
    static_assert(kChunks * 16 * (FQ == 2 ? 2 : 1) <= 152 * 1024, "the stage rings of the resident workgroups do not fit the LDS of a compute unit");
};

// s_waitcnt vmcnt(N): at most N vector memory operations of this wave still outstanding
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// Scheduling hints for one MFMA step: after each of its NM MFMAs, an even share of DS LDS reads and VM loads.
template <int I, int NM, int DS, int VM>
__device__ __forceinline__ void tile_interleave() {
    if constexpr (I < NM) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        constexpr int ds = DS * (I + 1) / NM - DS * I / NM, vm = VM * (I + 1) / NM - VM * I / NM;
        if constexpr (ds > 0) __builtin_amdgcn_sched_group_barrier(0x100, ds, 0);
        if constexpr (vm > 0) __builtin_amdgcn_sched_group_barrier(0x020, vm, 0);
        tile_interleave<I + 1, NM, DS, VM>();
    }
}

// Every wave fetches 8 of a stage's 32 rows of both operands: 4 load instructions for R and FQ for Q.
// Columns past the end of an operand are clamped onto its last chunk (valid memory; the caller never stores what they
// produce).  The caller guarantees that both operands have a whole number of stages of rows (zero rows at the end).
template <int FQ>
struct TileSource {
    const u32x4_t* p[4 + FQ];
    size_t step[4 + FQ];    // chunks from one stage to the next
};

// r0 / q0: first column of the tile in R / Q; nr / nq: their numbers of columns (multiples of 8); strides in chunks.
template <int FQ>
__device__ __forceinline__ TileSource<FQ> tile_source(const u32x4_t* __restrict__ R, int r0, int nr, size_t r_stride,
                                                      const u32x4_t* __restrict__ Q, int q0, int nq, size_t q_stride) {
    TileSource<FQ> src;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int krow = 8 * wave + 2 * i + (lane >> 5);                 // row of the stage's 32
        const int c = (lane & 31) ^ ((krow & 3) << 2);
        src.p[i] = R + size_t(krow) * r_stride + min(r0 / 8 + c, nr / 8 - 1);
        src.step[i] = 32 * r_stride;
    }
    constexpr int QC = 8 * FQ, QROWS = 64 / QC;                          // chunks per row of the Q stage, rows per load
#pragma unroll
    for (int i = 0; i < FQ; ++i) {
        const int krow = 8 * wave + QROWS * i + lane / QC;
        const int c = (lane % QC) ^ ((krow & 3) << 2);
        src.p[4 + i] = Q + size_t(krow) * q_stride + min(q0 / 8 + c, nq / 8 - 1);
        src.step[4 + i] = 32 * q_stride;
    }
    return src;
}

// acc[a][q] += (R columns [128 wy + 32 a, +32))^T (Q columns [32 FQ wx + 32 q, +32)) over nst >= 1 stages of 32 rows.
// NB: LDS stage buffers (NB - 2 stages are in flight while one is consumed and one is awaited).
// Called by all 256 threads; starts and ends with every LDS buffer free (a workgroup barrier closes the loop).
template <int NB, int FQ>
__device__ __forceinline__ void tile_mainloop(u32x4_t* __restrict__ lds, const TileSource<FQ>& src, int nst, f32x16_t (&acc)[4][FQ]) {
    typedef TileLds<NB, FQ> L;
    typedef __attribute__((ext_vector_type(4))) short s16x4_t;
    typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
    constexpr int NL = 4 + FQ;                                        // loads of one stage by one wave
    constexpr int NM = 4 * FQ;                                        // MFMAs of one step
    constexpr int READS = 2 * (4 + FQ);                               // LDS reads of one step's fragments
    constexpr int QW = 64 * FQ;                                       // elements in a row of the Q stage
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wy = wave >> 1, wx = wave & 1;
    auto issue = [&](int stage, int buf) {
        stage = min(stage, nst - 1);                                  // past the end: the last stage once more, into a free buffer
        u32x4_t* const dst = lds + buf * L::kStage + wave * 256;      // 8 rows of R: 8 x 32 chunks
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src.p[i] + stage * src.step[i]),
                                             (__attribute__((address_space(3))) void*)(dst + i * 64), 16, 0, 0);
        u32x4_t* const dq = lds + buf * L::kStage + L::kStageR + wave * (64 * FQ);      // 8 rows of Q: 8 x 8 FQ chunks
#pragma unroll
        for (int i = 0; i < FQ; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src.p[4 + i] + stage * src.step[4 + i]),
                                             (__attribute__((address_space(3))) void*)(dq + i * 64), 16, 0, 0);
    };
    u32x4_t fr[2][4], fq[2][FQ];
    // fragment addresses inside a stage buffer in 16-bit elements, for the two MFMA steps of a stage and the two reads
    // of a fragment: this lane's row and column inside the 4 x 16 block, then the fragment's (swizzled) chunk group
    int off_r[2][2], off_q[2][2], frag_r[4], frag_q[FQ];
    {
        const int G = lane >> 4, p = lane & 15, kk = (p >> 2) & 3;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int k = 16 * u + 8 * (G >> 1) + 4 * h + (p >> 2);          // k % 4 == kk
                const int col = 16 * (G & 1) + 4 * (p & 3);                       // within a fragment's 32 columns
                off_r[u][h] = k * 256 + col;
                off_q[u][h] = L::kStageR * 8 + k * QW + col;
            }
#pragma unroll
        for (int f = 0; f < 4; ++f) frag_r[f] = 8 * ((16 * wy + 4 * f) ^ (kk << 2));
#pragma unroll
        for (int f = 0; f < FQ; ++f) frag_q[f] = 8 * ((4 * FQ * wx + 4 * f) ^ (kk << 2));
    }
    auto read_frag = [&](const short* base, int o0, int o1) {
        const u32x2_t lo = __builtin_bit_cast(u32x2_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(base + o0)));
        const u32x2_t hi = __builtin_bit_cast(u32x2_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(base + o1)));
        return u32x4_t{lo.x, lo.y, hi.x, hi.y};
    };
    auto frags = [&](int buf, int u, int set) {
        const short* base = reinterpret_cast<const short*>(lds + buf * L::kStage);
#pragma unroll
        for (int f = 0; f < 4; ++f) fr[set][f] = read_frag(base, off_r[u][0] + frag_r[f], off_r[u][1] + frag_r[f]);
#pragma unroll
        for (int f = 0; f < FQ; ++f) fq[set][f] = read_frag(base, off_q[u][0] + frag_q[f], off_q[u][1] + frag_q[f]);
    };
    auto mfmas = [&](int set) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int q = 0; q < FQ; ++q) Bf16::mma(fr[set][a], fq[set][q], acc[a][q]);
    };
    for (int d = 0; d < NB - 1; ++d) issue(d, d);
    wait_vmcnt<NL * (NB - 2)>();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    int cur = 0, load_buf = NB - 1;
    frags(0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    for (int s = 0; s < nst; ++s) {
        const int nxt = cur + 1 == NB ? 0 : cur + 1;
        // first MFMA step of the stage: the fragments of its second step and this wave's loads of the stage NB - 1
        // ahead ride between the MFMAs, spread evenly
        frags(cur, 1, 1);
        issue(s + NB - 1, load_buf);
        mfmas(0);
        tile_interleave<0, NM, READS, NL>();
        __builtin_amdgcn_sched_barrier(0);
        wait_vmcnt<NL * (NB - 2)>();                                 // stage s + 1 has landed (the younger ones stay in flight)
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // second step: the fragments of the next stage's first step ride between the MFMAs
        frags(nxt, 0, 0);
        mfmas(1);
        tile_interleave<0, NM, READS, 0>();
        __builtin_amdgcn_sched_barrier(0);
        cur = nxt;
        load_buf = load_buf + 1 == NB ? 0 : load_buf + 1;
    }
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
}

}  // namespace pamm
