// Host-side planning: tile shapes and workspace layout, shared by the workspace queries and the launchers.
#pragma once

#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

#include "../../include/pamm.h"

namespace pamm {

constexpr int64_t kMaxGenerators = 16384;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int elem_bytes(pamm_dtype dt) { return dt == PAMM_BF16 ? 2 : 4; }
inline int per_chunk(pamm_dtype dt) { return dt == PAMM_BF16 ? 8 : 4; }

inline bool dtype_ok(pamm_dtype dt) { return dt == PAMM_F32 || dt == PAMM_BF16; }

// Tuning overrides for experiments (read on every call; unset or invalid = use the built-in heuristic):
//   PAMM_SCORE_TT    token fragments per wave in k_score (1 or 2)
//   PAMM_PIECE_ROWS  list positions per chunk in k_contract (a multiple of 16, 16..4096)
inline int env_int(const char* name) {
    const char* v = getenv(name);
    return v ? atoi(v) : 0;
}

// ------------------------------------------------------------------------------------ compress

struct CompressPlan {
    int tg;          // 32-generator fragments per wave (1, 2, 4 or 8): a column block holds 32*tg generators
    int tt;          // 32-token fragments per wave (1 or 2): a workgroup of 4 waves holds 128*tt tokens
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
    int tg = 1;
    while (tg < 8 && 32 * tg < k) tg *= 2;
    p->tg = tg;
    p->ncb = int((k + 32 * tg - 1) / (32 * tg));
    // two token fragments per wave halve the LDS reads per MFMA; use them once the grid still covers the chip
    int64_t tiles2 = (b + 255) / 256;
    p->tt = (tiles2 * p->ncb >= 512) ? 2 : 1;
    const int tt_env = env_int("PAMM_SCORE_TT");
    if (tt_env == 1 || tt_env == 2) p->tt = tt_env;
    p->row_tiles = (b + 128 * p->tt - 1) / (128 * p->tt);
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
    int piece_rows;       // P: the sorted row list is cut into chunks of P positions (a multiple of 16)
    int64_t chunks;       // ceil(b / P)
    int64_t nslots;       // upper bound on piece numbers: chunks + k
    int col_groups;       // ceil(m / 512): one wave covers 512 columns of a row
    int64_t kpad;         // k rounded up to a whole number of MFMA steps (16 generators for bf16, 8 for fp32)
    size_t off_perm, off_alpha, off_key, off_sbase, off_snum, off_partial, off_ct, off_bt, total;
};

inline pamm_status plan_grad(int64_t b, int64_t n, int64_t k, int64_t m, pamm_dtype dt, GradPlan* p) {
    if (!dtype_ok(dt)) return PAMM_ERR_UNSUPPORTED;
    if (b < 1 || n < 1 || m < 1 || k < 1 || b >= (int64_t(1) << 31) || n >= (int64_t(1) << 31) || m >= (int64_t(1) << 31))
        return PAMM_ERR_INVALID_ARG;
    if (k > kMaxGenerators) return PAMM_ERR_UNSUPPORTED;
    if (n % per_chunk(dt) != 0 || m % per_chunk(dt) != 0) return PAMM_ERR_UNSUPPORTED;
    p->col_groups = int((m + 511) / 512);
    // One wave per (chunk, column group).  All waves carry the same load, so the best grid is a single round
    // that fits the chip: ~14 waves per CU (16 fit at the kernel's register count).
    int64_t P = (b * p->col_groups + 3583) / 3584;
    P = (P + 15) / 16 * 16;
    if (P < 16) P = 16;
    if (P > 4096) P = 4096;
    const int p_env = env_int("PAMM_PIECE_ROWS");
    if (p_env >= 16 && p_env <= 4096 && p_env % 16 == 0) P = p_env;
    p->piece_rows = int(P);
    p->chunks = (b + P - 1) / P;
    p->nslots = p->chunks + k;
    const int64_t step = 2 * per_chunk(dt);
    p->kpad = (k + step - 1) / step * step;
    size_t o = 0;
    p->off_perm = o;    o = align_up(o + size_t(b) * 4, 256);
    p->off_alpha = o;   o = align_up(o + size_t(b) * 4, 256);
    p->off_key = o;     o = align_up(o + size_t(b) * 4, 256);
    p->off_sbase = o;   o = align_up(o + size_t(k) * 4, 256);
    p->off_snum = o;    o = align_up(o + size_t(k) * 4, 256);
    p->off_partial = o; o = align_up(o + size_t(p->nslots) * size_t(m) * 4, 256);
    p->off_ct = o;      o = align_up(o + size_t(n) * size_t(p->kpad) * elem_bytes(dt), 256);
    p->off_bt = o;      o = align_up(o + size_t(m) * size_t(p->kpad) * elem_bytes(dt), 256);
    p->total = o;
    return PAMM_OK;
}

}  // namespace pamm
