// Host-side planning: tile shapes and workspace layout, shared by the workspace queries and the launchers.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "../../include/pamm.h"

namespace pamm {

constexpr int64_t kMaxGenerators = 16384;
constexpr int64_t kNumCU = 256;            // compute units of the MI355X

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int elem_bytes(pamm_dtype dt) { return dt == PAMM_BF16 ? 2 : 4; }
inline int per_chunk(pamm_dtype dt) { return dt == PAMM_BF16 ? 8 : 4; }

inline bool dtype_ok(pamm_dtype dt) { return dt == PAMM_F32 || dt == PAMM_BF16; }

// Overrides of the built-in launch heuristics, set only through the test hook pamm_debug_set_plan (0 = heuristic).
// Product calls never read the environment; tests use the hook to reach the kernel variants and grid decompositions
// that the heuristics do not pick at the shapes they run.
//   score_tg       32-generator fragments per wave in k_score (1, 2, 4 or 8; at most what k allows)
//   score_nw       waves per workgroup in k_score (2, 4 or 8)
//   piece_rows     list positions per chunk in k_contract (a multiple of 16, 16..4096)
//   contract_w     512-column groups per wave in k_contract (1..3)
//   sort_one_rows  largest b sorted by the single-workgroup kernel (1..16384)
//   small_tiles    1: never take the big-tile kernel of the small product (k_ctb_big); 2: take it with 256 x 256 tiles
extern pamm_debug_plan g_plan_override;

// ------------------------------------------------------------------------------------ compress

struct CompressPlan {
    int tg;          // 32-generator fragments per wave (1, 2, 4 or 8): a column block holds 32*tg generators
    int tt;          // 32-token fragments per wave (always 1: two were measured slower than twice the waves)
    int nw;          // waves per workgroup (2, 4 or 8): a workgroup holds 32*tt*nw tokens
    int ncb;         // column blocks = ceil(k / (32*tg))
    int64_t row_tiles;
    // workspace offsets (bytes)
    size_t off_idx, off_rn, off_cn2, off_hash, off_cand, total;
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
    const int tg_forced = g_plan_override.score_tg;
    if ((tg_forced == 1 || tg_forced == 2 || tg_forced == 4 || tg_forced == 8) && tg_forced <= tg_max) tg = tg_forced;
    const int nw_forced = g_plan_override.score_nw;
    if (nw_forced == 2 || nw_forced == 4 || nw_forced == 8) nw = nw_forced;
    p->tg = tg;
    p->ncb = int(blocks(tg));
    p->tt = 1;
    p->nw = nw;
    const int64_t tile_tokens = 32 * p->tt * p->nw;
    p->row_tiles = (b + tile_tokens - 1) / tile_tokens;
    size_t o = 0;
    p->off_idx = o;  o = align_up(o + size_t(k) * 4, 256);
    p->off_rn = o;   o = align_up(o + size_t(k) * 4, 256);
    p->off_cn2 = o;  o = align_up(o + size_t(k) * 8, 256);
    p->off_hash = o; o = align_up(o + size_t(k) * 8, 256);
    p->off_cand = o; o = align_up(o + size_t(b) * size_t(p->ncb) * 32, 256);
    p->total = o;
    return PAMM_OK;
}

// ---------------------------------------------------------------------------------------- grad

struct GradPlan {
    int p_fixed;          // chunk size forced by the test hook (0: chosen on the device from the length of the list)
    int64_t chunks;       // upper bound on the number of chunks the sorted list is cut into
    int64_t nslots;       // upper bound on piece numbers: chunks + k
    int col_groups;       // ceil(m / 512)
    int sort_one_rows;    // batches up to this many rows are sorted by one workgroup in one kernel
    int wave_groups;      // W: 512-column groups per wave (1..3); a workgroup of 4 waves covers 4*W groups of a row
    int wg_cols;          // workgroups side by side along a row: ceil(col_groups / (4*W))
    int64_t kpad;         // k rounded up to a whole number of k_ctb stages (32 generators for bf16, 16 for fp32)
    bool big_tiles;       // C^T Btilde on 256 x 128 tiles (k_ctb_big): bf16, many generators, a large weight gradient
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
    const int w_forced = g_plan_override.contract_w;
    if (w_forced >= 1 && w_forced <= 3) W = w_forced;
    p->wave_groups = W;
    const int so_forced = g_plan_override.sort_one_rows;
    p->sort_one_rows = (so_forced >= 1 && so_forced <= 16384) ? so_forced : 8192;
    p->wg_cols = (p->col_groups + 4 * W - 1) / (4 * W);
    // One workgroup per (chunk, 4*W column groups).  All workgroups carry the same load, and measured on the
    // MI355X the contraction runs best as one even round: exactly one workgroup per CU (256 CUs), i.e. few, long
    // chunks (4 waves per CU, each with >= 12 KiB of dY in flight).  The list only holds the rows with a non-zero
    // weight, L <= b of them, so the chunk size P = clamp(roundup16(L * wg_cols / 256), 16, 4096) is set on the
    // device; whatever L is, that gives at most max(ceil(256 / wg_cols), ceil(b / 4096)) + 1 chunks.
    const int p_forced = g_plan_override.piece_rows;
    p->p_fixed = (p_forced >= 16 && p_forced <= 4096 && p_forced % 16 == 0) ? p_forced : 0;
    if (p->p_fixed) {
        p->chunks = (b + p->p_fixed - 1) / p->p_fixed;
    } else {
        const int64_t even = (kNumCU + p->wg_cols - 1) / p->wg_cols, longest = (b + 4095) / 4096;
        p->chunks = (even > longest ? even : longest) + 1;
    }
    p->nslots = p->chunks + k;
    // The product C^T Btilde runs on big tiles (k_ctb_big) where the matrix cores are its limit: bf16, at least 512
    // generators (with fewer the product is bound by the write of the result, which the small tiles overlap better) and
    // a result of at least two 256 x 256 blocks per compute unit.
    p->big_tiles = dt == PAMM_BF16 && k >= 512 && ((n + 255) / 256) * ((m + 255) / 256) >= 2 * kNumCU && g_plan_override.small_tiles != 1;
    const int64_t stage_gens = 4 * per_chunk(dt);      // generators per stage: 32 (bf16) or 16 (fp32)
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

// ------------------------------------------------------------------------- argument checks of the entry points
// All of them run on the host before anything is enqueued; kept here, free of device code, so that a plain CPU build
// can run them under the address and undefined-behaviour sanitizers.

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

inline pamm_status check_compress_args(const void* X, int64_t b, int64_t n, int64_t k, pamm_dtype dt, const void* C, const void* f,
                                       const void* alpha, const void* ws, size_t ws_bytes, CompressPlan* pl) {
    pamm_status st = plan_compress(b, n, k, dt, pl);
    if (st != PAMM_OK) return st;
    if (!X || !C || !f || !alpha) return PAMM_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(C) || !aligned16(f) || !aligned16(alpha)) return PAMM_ERR_INVALID_ARG;
    if (!ws || ws_bytes < pl->total) return PAMM_ERR_WORKSPACE;
    if (!aligned16(ws)) return PAMM_ERR_INVALID_ARG;
    return PAMM_OK;
}

// eps -> keep = 1 - eps^2 (negative: the condition cannot drop anything and is switched off)
inline pamm_status keep_of(float eps, double* keep) {
    if (!(eps >= 0.f)) return PAMM_ERR_INVALID_ARG;          // negative or NaN
    *keep = eps < 1.f ? 1.0 - double(eps) * double(eps) : -1.0;
    return PAMM_OK;
}

inline pamm_status check_contract_args(const void* f, const void* alpha, const void* dY, int64_t b, int64_t k, int64_t m,
                                       pamm_dtype dt, const void* Btilde, const void* ws, size_t ws_bytes, GradPlan* pl) {
    pamm_status st = plan_grad(b, per_chunk(dtype_ok(dt) ? dt : PAMM_F32), k, m, dt, pl);   // n does not enter what is used
    if (st != PAMM_OK) return st;
    if (k > b) return PAMM_ERR_INVALID_ARG;
    if (!f || !alpha || !dY || !Btilde) return PAMM_ERR_INVALID_ARG;
    if (!aligned16(f) || !aligned16(alpha) || !aligned16(dY) || !aligned16(Btilde)) return PAMM_ERR_INVALID_ARG;
    if (!ws || ws_bytes < pl->total) return PAMM_ERR_WORKSPACE;
    if (!aligned16(ws)) return PAMM_ERR_INVALID_ARG;
    return PAMM_OK;
}

inline pamm_status check_grad_args(const void* C, const void* f, const void* alpha, const void* dY, int64_t b, int64_t n, int64_t k,
                                   int64_t m, pamm_dtype dt, pamm_dtype out_dt, pamm_layout layout, const void* dW, const void* ws,
                                   size_t ws_bytes, GradPlan* pl) {
    pamm_status st = plan_grad(b, n, k, m, dt, pl);
    if (st != PAMM_OK) return st;
    if (!dtype_ok(out_dt) || (layout != PAMM_DW_N_BY_M && layout != PAMM_DW_M_BY_N)) return PAMM_ERR_UNSUPPORTED;
    if (out_dt == PAMM_BF16 && (((layout == PAMM_DW_M_BY_N) ? n : m) & 1)) return PAMM_ERR_UNSUPPORTED;   // pairs of columns
    if (k > b) return PAMM_ERR_INVALID_ARG;
    if (!C || !f || !alpha || !dY || !dW) return PAMM_ERR_INVALID_ARG;
    if (!aligned16(C) || !aligned16(f) || !aligned16(alpha) || !aligned16(dY) || !aligned16(dW)) return PAMM_ERR_INVALID_ARG;
    if (!ws || ws_bytes < pl->total) return PAMM_ERR_WORKSPACE;
    if (!aligned16(ws)) return PAMM_ERR_INVALID_ARG;
    return PAMM_OK;
}

// -------------------------------------------------------------------------------------- sketch

constexpr int64_t kMaxSketch = 128;        // widest sketch: four 32-wide fragments next to four of dY in a wave's registers

inline pamm_status check_sketch_sizes(int64_t b, int64_t n, int64_t r, pamm_dtype dt) {
    if (!dtype_ok(dt)) return PAMM_ERR_UNSUPPORTED;
    if (b < 1 || n < 1 || r < 1 || r > b || b >= (int64_t(1) << 31) || n >= (int64_t(1) << 31)) return PAMM_ERR_INVALID_ARG;
    if (r > kMaxSketch || n % per_chunk(dt) != 0 || r % per_chunk(dt) != 0) return PAMM_ERR_UNSUPPORTED;
    return PAMM_OK;
}

// pamm_sketch_grad: G = S^T dY in partial rows (one per sketch column and chunk of tokens), then the small product of
// ApproxMM with P^T in the place of C and the sketch columns in the place of the generators.
struct SketchGradPlan {
    GradPlan g;           // what the small product reads: kpad, big_tiles and the offsets of sbase, snum, partial, ct, bt
    int nr;               // 32-wide fragments of the sketch: ceil(r / 32)
    int col_groups;       // a workgroup takes 512 (bf16) or 256 (fp32) columns of dY
    int64_t chunk_rows;   // tokens per chunk, a multiple of 32
    int64_t chunks;
    size_t off_zero, total;
};

inline pamm_status plan_sketch_grad(int64_t b, int64_t n, int64_t r, int64_t m, pamm_dtype dt, SketchGradPlan* p) {
    pamm_status st = check_sketch_sizes(b, n, r, dt);
    if (st != PAMM_OK) return st;
    if (m < 1 || m >= (int64_t(1) << 31)) return PAMM_ERR_INVALID_ARG;
    if (m % per_chunk(dt) != 0) return PAMM_ERR_UNSUPPORTED;
    p->nr = int((r + 31) / 32);
    const int64_t group = dt == PAMM_BF16 ? 512 : 256;      // columns of dY per workgroup
    p->col_groups = int((m + group - 1) / group);
    // At most two workgroups per compute unit in all, as near to that as whole chunks allow: the LDS ring admits one
    // workgroup per compute unit at a time, all carry the same load, and a few left over would cost a third round.
    int64_t want = 2 * kNumCU / p->col_groups;
    want = want < 1 ? 1 : want;
    int64_t rows = (b + want - 1) / want;
    rows = (rows + 31) / 32 * 32;
    p->chunk_rows = rows < 128 ? 128 : rows;
    p->chunks = (b + p->chunk_rows - 1) / p->chunk_rows;
    GradPlan& g = p->g;
    g = GradPlan{};
    g.big_tiles = false;
    const int64_t stage_gens = 4 * per_chunk(dt);      // the small product's stages: 32 (bf16) or 16 (fp32) sketch columns
    g.kpad = (r + stage_gens - 1) / stage_gens * stage_gens;
    size_t o = 0;
    p->off_zero = o;    o = align_up(o + 16, 256);
    g.off_sbase = o;    o = align_up(o + size_t(r) * 4, 256);
    g.off_snum = o;     o = align_up(o + size_t(r) * 4, 256);
    g.off_partial = o;  o = align_up(o + size_t(r) * size_t(p->chunks) * size_t(m) * 4, 256);
    g.off_ct = o;       o = align_up(o + size_t(n) * size_t(g.kpad) * elem_bytes(dt), 256);
    g.off_bt = o;       o = align_up(o + size_t(m) * size_t(g.kpad) * elem_bytes(dt), 256);
    g.off_list = g.off_hdr = g.off_table = 0;      // not used
    g.total = o;
    p->total = o;
    return PAMM_OK;
}

inline pamm_status check_sketch_args(const void* X, const void* Pt, int64_t b, int64_t n, int64_t r, pamm_dtype dt, const void* S) {
    pamm_status st = check_sketch_sizes(b, n, r, dt);
    if (st != PAMM_OK) return st;
    if (!X || !Pt || !S) return PAMM_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(Pt) || !aligned16(S)) return PAMM_ERR_INVALID_ARG;
    return PAMM_OK;
}

inline pamm_status check_sketch_grad_args(const void* Pt, const void* S, const void* dY, int64_t b, int64_t n, int64_t r, int64_t m,
                                          pamm_dtype dt, const void* dW, const void* ws, size_t ws_bytes, SketchGradPlan* pl) {
    pamm_status st = plan_sketch_grad(b, n, r, m, dt, pl);
    if (st != PAMM_OK) return st;
    if (!Pt || !S || !dY || !dW) return PAMM_ERR_INVALID_ARG;
    if (!aligned16(Pt) || !aligned16(S) || !aligned16(dY) || !aligned16(dW)) return PAMM_ERR_INVALID_ARG;
    if (!ws || ws_bytes < pl->total) return PAMM_ERR_WORKSPACE;
    if (!aligned16(ws)) return PAMM_ERR_INVALID_ARG;
    return PAMM_OK;
}

}  // namespace pamm
