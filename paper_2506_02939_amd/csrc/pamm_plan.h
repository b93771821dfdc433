// Host-side planning: tile shapes and workspace layout, shared by the workspace queries and the launchers.
#pragma once

#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

#include "../../include/pamm.h"

namespace pamm {

constexpr int64_t kMaxGenerators = 16384;
constexpr int64_t kNumCU = 256;            // compute units of the MI355X

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int elem_bytes(pamm_dtype dt) { return dt == PAMM_BF16 ? 2 : 4; }
inline int per_chunk(pamm_dtype dt) { return dt == PAMM_BF16 ? 8 : 4; }

inline bool dtype_ok(pamm_dtype dt) { return dt == PAMM_F32 || dt == PAMM_BF16; }

// Tuning overrides for experiments (read on every call; unset or invalid = use the built-in heuristic):
//   PAMM_SCORE_TG    32-generator fragments per wave in k_score (1, 2, 4 or 8; at most what k allows)
//   PAMM_SCORE_NW    waves per workgroup in k_score (2, 4 or 8)
//   PAMM_PIECE_ROWS  list positions per chunk in k_contract (a multiple of 16, 16..4096)
//   PAMM_CONTRACT_W  512-column groups per wave in k_contract (1..3)
//   PAMM_SORT_ONE    largest b sorted by the single-workgroup kernel (1..16384)
inline int env_int(const char* name) {
    const char* v = getenv(name);
    return v ? atoi(v) : 0;
}

// ------------------------------------------------------------------------------------ compress

struct CompressPlan {
    int tg;          // 32-generator fragments per wave (1, 2, 4 or 8): a column block holds 32*tg generators
    int tt;          // 32-token fragments per wave (always 1: two were measured slower than twice the waves)
    int nw;          // waves per workgroup (2, 4 or 8): a workgroup holds 32*tt*nw tokens
    int ncb;         // column blocks = ceil(k / (32*tg))
    int64_t row_tiles;
    // workspace offsets (bytes)
    size_t off_idx, off_inv, off_cn2, off_hash, off_cand, total;
};

inline pamm_status plan_compress(int64_t b, int64_t n, int64_t k, pamm_dtype dt, CompressPlan* p) {
    if (!dtype_ok(dt)) return PAMM_ERR_UNSUPPORTED;
    if (b < 1 || n < 1 || k < 1 || k > b || b >= (int64_t(1) << 31) || n >= (int64_t(1) << 31)) return PAMM_ERR_INVALID_ARG;
    if (k > kMaxGenerators) return PAMM_ERR_UNSUPPORTED;
    if (n % per_chunk(dt) != 0) return PAMM_ERR_UNSUPPORTED;
    // A workgroup scores 32*nw tokens (nw waves, 32 each) against a column block of 32*tg generators.  Wanted, in
    // this order: enough workgroups to give every CU one (at least 224), at least four waves in each (one per SIMD,
    // better eight), and column blocks as wide as the generators allow (fewer passes over X; with a single block
    // the kernel also takes the final decision).  When the widest block leaves CUs idle or SIMDs empty (few tokens,
    // many generators), narrower blocks are tried, down to a quarter of the widest.
    int tg_max = 1;
    while (tg_max < 8 && 32 * tg_max < k) tg_max *= 2;
    auto blocks = [&](int tg) { return (k + 32 * tg - 1) / (32 * tg); };
    auto tiles = [&](int nw) { return (b + 32 * nw - 1) / (32 * nw); };
    int tg = tg_max, nw = 0;
    for (int t = tg_max; t >= 1 && t * 4 >= tg_max && nw == 0; t /= 2)
        for (int w = 8; w >= 4 && nw == 0; w /= 2)
            if (tiles(w) * blocks(t) >= 224) { tg = t; nw = w; }
    if (nw == 0) {               // nothing fills the chip: widest blocks, as many waves as still give every CU a workgroup
        nw = 8;
        while (nw > 2 && tiles(nw) * blocks(tg) < 224) nw /= 2;
    }
    const int tg_env = env_int("PAMM_SCORE_TG");
    if ((tg_env == 1 || tg_env == 2 || tg_env == 4 || tg_env == 8) && tg_env <= tg_max) tg = tg_env;
    const int nw_env = env_int("PAMM_SCORE_NW");
    if (nw_env == 2 || nw_env == 4 || nw_env == 8) nw = nw_env;
    p->tg = tg;
    p->ncb = int(blocks(tg));
    p->tt = 1;
    p->nw = nw;
    const int64_t tile_tokens = 32 * p->tt * p->nw;
    p->row_tiles = (b + tile_tokens - 1) / tile_tokens;
    size_t o = 0;
    p->off_idx = o;  o = align_up(o + size_t(k) * 4, 256);
    p->off_inv = o;  o = align_up(o + size_t(k) * 4, 256);
    p->off_cn2 = o;  o = align_up(o + size_t(k) * 8, 256);
    p->off_hash = o; o = align_up(o + size_t(k) * 8, 256);
    p->off_cand = o; o = align_up(o + size_t(b) * size_t(p->ncb) * 32, 256);
    p->total = o;
    return PAMM_OK;
}

// ---------------------------------------------------------------------------------------- grad

struct GradPlan {
    int p_fixed;          // chunk size forced by PAMM_PIECE_ROWS (0: chosen on the device from the length of the list)
    int64_t chunks;       // upper bound on the number of chunks the sorted list is cut into
    int64_t nslots;       // upper bound on piece numbers: chunks + k
    int col_groups;       // ceil(m / 512)
    int sort_one_rows;    // batches up to this many rows are sorted by one workgroup in one kernel
    int wave_groups;      // W: 512-column groups per wave (1..3); a workgroup of 4 waves covers 4*W groups of a row
    int wg_cols;          // workgroups side by side along a row: ceil(col_groups / (4*W))
    int64_t kpad;         // k rounded up to a whole number of k_ctb stages (32 generators for bf16, 16 for fp32)
    int slice_rows;       // rows per slice of the counting sort (1024 or 4096)
    int64_t nslices;      // ceil(b / slice_rows)
    size_t off_list, off_hdr, off_sbase, off_snum, off_table, off_partial, off_ct, off_bt, total;
};

inline pamm_status plan_grad(int64_t b, int64_t n, int64_t k, int64_t m, pamm_dtype dt, GradPlan* p) {
    if (!dtype_ok(dt)) return PAMM_ERR_UNSUPPORTED;
    if (b < 1 || n < 1 || m < 1 || k < 1 || b >= (int64_t(1) << 31) || n >= (int64_t(1) << 31) || m >= (int64_t(1) << 31))
        return PAMM_ERR_INVALID_ARG;
    if (k > kMaxGenerators) return PAMM_ERR_UNSUPPORTED;
    if (n % per_chunk(dt) != 0 || m % per_chunk(dt) != 0) return PAMM_ERR_UNSUPPORTED;
    p->col_groups = int((m + 511) / 512);
    int W = (p->col_groups + 3) / 4;
    W = W < 1 ? 1 : (W > 3 ? 3 : W);
    const int w_env = env_int("PAMM_CONTRACT_W");
    if (w_env >= 1 && w_env <= 3) W = w_env;
    p->wave_groups = W;
    const int so_env = env_int("PAMM_SORT_ONE");
    p->sort_one_rows = (so_env >= 1 && so_env <= 16384) ? so_env : 8192;
    p->wg_cols = (p->col_groups + 4 * W - 1) / (4 * W);
    // One workgroup per (chunk, 4*W column groups).  All workgroups carry the same load, and measured on the
    // MI355X the contraction runs best as one even round: exactly one workgroup per CU (256 CUs), i.e. few, long
    // chunks (4 waves per CU, each with >= 12 KiB of dY in flight).  The list only holds the rows with a non-zero
    // weight, L <= b of them, so the chunk size P = clamp(roundup16(L * wg_cols / 256), 16, 4096) is set on the
    // device; whatever L is, that gives at most max(ceil(256 / wg_cols), ceil(b / 4096)) + 1 chunks.
    const int p_env = env_int("PAMM_PIECE_ROWS");
    p->p_fixed = (p_env >= 16 && p_env <= 4096 && p_env % 16 == 0) ? p_env : 0;
    if (p->p_fixed) {
        p->chunks = (b + p->p_fixed - 1) / p->p_fixed;
    } else {
        const int64_t even = (kNumCU + p->wg_cols - 1) / p->wg_cols, longest = (b + 4095) / 4096;
        p->chunks = (even > longest ? even : longest) + 1;
    }
    p->nslots = p->chunks + k;
    const int64_t stage_gens = 4 * per_chunk(dt);      // generators per k_ctb stage: 32 (bf16) or 16 (fp32)
    p->kpad = (k + stage_gens - 1) / stage_gens * stage_gens;
    // Counting sort of the rows by generator: short slices spread the scattered list writes over many CUs, but every
    // slice's workgroup sums the whole table of slice histograms (slices x k entries), so that table must stay small.
    p->slice_rows = ((b + 1023) / 1024) * k <= 4096 ? 1024 : 4096;
    p->nslices = (b + p->slice_rows - 1) / p->slice_rows;
    size_t o = 0;
    p->off_list = o;    o = align_up(o + size_t(b + 16) * 16, 256);     // 16-byte entries, padded to a multiple of 16 entries
    p->off_hdr = o;     o = align_up(o + 16, 256);                      // list length and chunk size, written by the grouping
    p->off_sbase = o;   o = align_up(o + size_t(k) * 4, 256);
    p->off_snum = o;    o = align_up(o + size_t(k) * 4, 256);
    p->off_table = o;   o = align_up(o + size_t(p->nslices) * size_t(k) * 4, 256);           // per-slice histograms
    p->off_partial = o; o = align_up(o + size_t(p->nslots) * size_t(m) * 4, 256);
    p->off_ct = o;      o = align_up(o + size_t(n) * size_t(p->kpad) * elem_bytes(dt), 256);
    p->off_bt = o;      o = align_up(o + size_t(m) * size_t(p->kpad) * elem_bytes(dt), 256);
    p->total = o;
    return PAMM_OK;
}

}  // namespace pamm
