// Main loop of a 256 x 256 tile of a product D = R Q^T of two bf16 operands whose contraction index is contiguous in
// memory (R: the operand that gives the rows of D, Q: the one that gives its columns), for the shapes where the matrix
// cores are the limit.  Used by the small product of ApproxMM (R = C^T, Q = Btilde^T, contraction over the generators).
//
// Workgroup = 4 waves in a 2 x 2 arrangement, each with a 128 x 128 part of the tile: 4 x 4 MFMA 32x32x16 accumulators
// (256 registers), one wave per SIMD.  The contraction index is walked in stages of 32 elements (4 chunks of 16 bytes
// per row, two MFMA steps); a stage of one operand is 16 KiB of LDS and each operand has a ring of them, filled by
// loads that go from global memory straight into LDS (no register hop: a wave has no registers to spare next to its
// accumulators, and nothing has to be waited for in the middle of the MFMA stream).  Such a load writes its 64 lanes'
// 16 bytes to consecutive LDS addresses, so the layout is chosen through WHICH chunk a lane fetches: 16 rows per
// instruction, row r keeps chunk c at position c ^ tile_swizzle(r), which makes the 16-byte fragment reads (32 rows,
// one chunk column) free of bank conflicts.  Inside an MFMA step the LDS reads of the next step's fragments and the
// loads of a later stage are issued one by one between the MFMAs (with one wave per SIMD nothing else hides
// their issue slots), and the only wait is the one before the workgroup barrier in the middle of every stage.
#pragma once

#include "pamm_device.h"

namespace pamm {

constexpr int kTileOperandChunks = 1024;           // one stage of one operand: 256 rows x 4 chunks (16 KiB)

template <int NBR, int NBQ>
struct TileLds {
    static constexpr int kChunks = (NBR + NBQ) * kTileOperandChunks;
    static_assert(kChunks * 16 <= 152 * 1024, "the stage rings do not fit the LDS of a compute unit next to the epilogue's own");
};

__device__ __forceinline__ int tile_swizzle(int r) { return ((r >> 1) & 3) ^ ((r >> 2) & 3); }

// s_waitcnt vmcnt(N): at most N vector memory operations of this wave still outstanding
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// Loading is split by operand: waves 0 and 1 fetch the rows of R (128 each), waves 2 and 3 those of Q, 8 load
// instructions of 16 rows per stage and wave.  Every wave counts its own outstanding loads, so the two operands can
// be fetched different distances ahead: an operand that streams from HBM needs a deep ring, one that sits in L2 a
// shallow one.  Lane L of an instruction takes row L/4 of its 16 rows and the chunk that belongs at position L%4.
// Rows past the end of an operand are clamped onto its last row (valid memory; the caller never stores what they
// produce).
struct TileSource {
    const u32x4_t* p[8];
};

__device__ __forceinline__ TileSource tile_source(const u32x4_t* __restrict__ R, int r0, int nr, size_t r_stride,
                                                  const u32x4_t* __restrict__ Q, int q0, int nq, size_t q_stride) {
    TileSource src;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = ((wave & 1) * 8 + i) * 16 + (lane >> 2);         // row of the operand's 256
        const int c = (lane & 3) ^ tile_swizzle(row);
        src.p[i] = wave < 2 ? R + size_t(min(r0 + row, nr - 1)) * r_stride + c : Q + size_t(min(q0 + row, nq - 1)) * q_stride + c;
    }
    return src;
}

// acc[a][q] += R rows [128 wy + 32 a, +32) x Q rows [128 wx + 32 q, +32) over nst >= 1 stages.  NBR / NBQ: LDS stage
// buffers of the two operands (a ring of NB lets NB - 2 stages be in flight while one is consumed and one is awaited).
// The walk over the contraction index starts at stage `rot` (0 <= rot < nst) and wraps around: a dot product does not
// care where it starts, and workgroups that share an operand through one L2 can be made to walk in step.
// Called by all 256 threads; starts and ends with every LDS buffer free (a workgroup barrier closes the loop).
template <int NBR, int NBQ>
__device__ __forceinline__ void tile_mainloop(u32x4_t* __restrict__ lds, const TileSource& src, int nst, int rot, f32x16_t (&acc)[4][4]) {
    constexpr int OP = kTileOperandChunks;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 31, g = lane >> 5;
    const int wy = wave >> 1, wx = wave & 1;
    const bool loads_r = wave < 2;                                   // uniform per wave
    u32x4_t* const ring_r = lds;
    u32x4_t* const ring_q = lds + NBR * OP;
    u32x4_t* const my_ring = (loads_r ? ring_r : ring_q) + (wave & 1) * 512;      // this wave's 128 rows of each buffer
    const int my_nb = loads_r ? NBR : NBQ;
    auto issue = [&](int stage, int buf) {
        stage = min(stage, nst - 1);                                 // past the end: the last stage once more, into a free buffer
        const int at = stage + rot - (stage + rot >= nst ? nst : 0);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src.p[i] + at * 4),
                                             (__attribute__((address_space(3))) void*)(my_ring + buf * OP + i * 64), 16, 0, 0);
    };
    // fragment addresses inside a buffer (chunks): row * 4 + swizzled chunk, for the two MFMA steps of a stage
    int off_r[2], off_q[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int ra = wy * 128 + r, rb = wx * 128 + r;              // + 32 f: the swizzle only looks at bits 1..3 of the row
        off_r[u] = ra * 4 + ((2 * u + g) ^ tile_swizzle(ra));
        off_q[u] = rb * 4 + ((2 * u + g) ^ tile_swizzle(rb));
    }
    u32x4_t fr[2][4], fq[2][4];
    auto frags = [&](int buf_r, int buf_q, int u, int set) {
        const u32x4_t* br = ring_r + buf_r * OP + off_r[u];
        const u32x4_t* bq = ring_q + buf_q * OP + off_q[u];
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            fr[set][f] = br[f * 128];
            fq[set][f] = bq[f * 128];
        }
    };
    auto mfmas = [&](int set) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int q = 0; q < 4; ++q) Bf16::mma(fr[set][a], fq[set][q], acc[a][q]);
    };
    auto wait_mine = [&]() {                                          // this wave's loads of the next stage have landed
        if (loads_r) wait_vmcnt<8 * (NBR - 2)>(); else wait_vmcnt<8 * (NBQ - 2)>();
    };
    // this wave's ring position of the stage being consumed / being loaded (my_nb - 1 ahead), and both operands' positions
    for (int d = 0; d < my_nb - 1; ++d) issue(d, d);
    wait_mine();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    int cur_r = 0, cur_q = 0, load_buf = my_nb - 1;
    frags(0, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    for (int s = 0; s < nst; ++s) {
        const int nxt_r = cur_r + 1 == NBR ? 0 : cur_r + 1, nxt_q = cur_q + 1 == NBQ ? 0 : cur_q + 1;
        // first MFMA step of the stage: the fragments of its second step and this wave's loads of the stage my_nb - 1
        // ahead ride between the MFMAs, one by one
        frags(cur_r, cur_q, 1, 1);
        issue(s + my_nb - 1, load_buf);
        mfmas(0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one MFMA,
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      // one LDS read
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one MFMA,
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);      // one load
        }
        __builtin_amdgcn_sched_barrier(0);
        wait_mine();                                                // stage s + 1 has landed (the younger ones stay in flight)
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // second step: the fragments of the next stage's first step ride between the MFMAs
        frags(nxt_r, nxt_q, 0, 0);
        mfmas(1);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        cur_r = nxt_r;
        cur_q = nxt_q;
        load_buf = load_buf + 1 == my_nb ? 0 : load_buf + 1;
    }
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
}

}  // namespace pamm
