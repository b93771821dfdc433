// Main loop of a 256 x 256 tile of a product D = R Q^T of two bf16 operands whose contraction index is contiguous in
// memory (R: the operand that gives the rows of D, Q: the one that gives its columns), for the shapes where the matrix
// cores are the limit.  Shared by the score kernel (R = generators, Q = tokens, contraction over the hidden dimension)
// and by the small product of ApproxMM (R = C^T, Q = Btilde^T, contraction over the generators).
//
// Workgroup = 4 waves in a 2 x 2 arrangement, each with a 128 x 128 part of the tile: 4 x 4 MFMA 32x32x16 accumulators
// (256 registers), one wave per SIMD.  The contraction index is walked in stages of 32 elements (4 chunks of 16 bytes
// per row, two MFMA steps); a stage of both operands is 32 KiB of LDS and kTileBuffers of them rotate, filled by
// loads that go from global memory straight into LDS (no register hop: a wave has no registers to spare next to its
// accumulators, and nothing has to be waited for in the middle of the MFMA stream).  Such a load writes its 64 lanes'
// 16 bytes to consecutive LDS addresses, so the layout is chosen through WHICH chunk a lane fetches: 16 rows per
// instruction, row r keeps chunk c at position c ^ tile_swizzle(r), which makes the 16-byte fragment reads (32 rows,
// one chunk column) free of bank conflicts.  Inside an MFMA step the LDS reads of the next step's fragments and the
// loads of the stage NB-1 ahead are issued one by one between the MFMAs (with one wave per SIMD nothing else hides
// their issue slots), and the only wait is the one before the workgroup barrier in the middle of every stage.
#pragma once

#include "pamm_device.h"

namespace pamm {

constexpr int kTileBuffers = 4;                   // LDS stage buffers (3 stages in flight while one is consumed)
constexpr int kTileStageChunks = 2048;            // 256 + 256 rows x 4 chunks
constexpr int kTileLdsBytes = kTileBuffers * kTileStageChunks * 16;

__device__ __forceinline__ int tile_swizzle(int r) { return ((r >> 1) & 3) ^ ((r >> 2) & 3); }

// s_waitcnt vmcnt(N): at most N vector memory operations of this wave still outstanding
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// Where the 8 load instructions of this lane's wave read from at stage 0: instruction i of wave w fills rows
// 16 (8 w + i) .. + 15 of the stage (rows 0..255: operand R, 256..511: operand Q), lane L the row L/4 of those and the
// chunk that belongs at position L%4.  Rows past the end of an operand are clamped onto its last row (valid memory;
// the caller never stores what they produce).
struct TileSource {
    const u32x4_t* p[8];
};

__device__ __forceinline__ TileSource tile_source(const u32x4_t* __restrict__ R, int r0, int nr, size_t r_stride,
                                                  const u32x4_t* __restrict__ Q, int q0, int nq, size_t q_stride) {
    TileSource src;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int row = (wave * 8 + i) * 16 + (lane >> 2);
        const int c = (lane & 3) ^ tile_swizzle(row);
        src.p[i] = row < 256 ? R + size_t(min(r0 + row, nr - 1)) * r_stride + c : Q + size_t(min(q0 + row - 256, nq - 1)) * q_stride + c;
    }
    return src;
}

// acc[a][q] += R rows [128 wy + 32 a, +32) x Q rows [128 wx + 32 q, +32) over nst stages, nst a multiple of kTileBuffers.
// Called by all 256 threads; starts and ends with every LDS buffer free (a workgroup barrier closes the loop).
__device__ __forceinline__ void tile_mainloop(u32x4_t* __restrict__ lds, const TileSource& src, int nst, f32x16_t (&acc)[4][4]) {
    constexpr int NB = kTileBuffers, STAGE = kTileStageChunks;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 31, g = lane >> 5;
    const int wy = wave >> 1, wx = wave & 1;
    auto issue = [&](int stage, int buf) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src.p[i] + stage * 4),
                                             (__attribute__((address_space(3))) void*)(lds + buf * STAGE + (wave * 8 + i) * 64), 16, 0, 0);
    };
    u32x4_t fr[2][4], fq[2][4];
    auto frags = [&](int buf, int u, int set) {
        const u32x4_t* base = lds + buf * STAGE;
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            const int ra = wy * 128 + 32 * f + r, rb = 256 + wx * 128 + 32 * f + r;
            fr[set][f] = base[ra * 4 + ((2 * u + g) ^ tile_swizzle(ra))];
            fq[set][f] = base[rb * 4 + ((2 * u + g) ^ tile_swizzle(rb))];
        }
    };
    auto mfmas = [&](int set) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int q = 0; q < 4; ++q) Bf16::mma(fr[set][a], fq[set][q], acc[a][q]);
    };
#pragma unroll
    for (int d = 0; d < NB - 1; ++d) issue(d, d);
    wait_vmcnt<8 * (NB - 2)>();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    frags(0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    for (int s0 = 0; s0 < nst; s0 += NB) {
#pragma unroll
        for (int bq = 0; bq < NB; ++bq) {
            const int s = s0 + bq;
            // first MFMA step of the stage: the fragments of its second step and the loads of stage s + NB - 1 ride between
            // the MFMAs (past the end the last stage is loaded once more, into a buffer nobody reads any more)
            frags(bq, 1, 1);
            issue(min(s + NB - 1, nst - 1), (bq + NB - 1) % NB);
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
            wait_vmcnt<8 * (NB - 2)>();                                 // stage s + 1 has landed (the younger ones stay in flight)
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            // second step: the fragments of the next stage's first step ride between the MFMAs
            frags((bq + 1) % NB, 0, 0);
            mfmas(1);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
}

}  // namespace pamm
