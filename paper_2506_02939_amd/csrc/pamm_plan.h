// Host-side planning: tile shapes and workspace layout, shared by the workspace queries and the launchers.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "../../include/pamm.h"

namespace pamm {

constexpr int64_t kMaxGenerators = 16384;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int elem_bytes(pamm_dtype dt) { return dt == PAMM_BF16 ? 2 : 4; }
inline int per_chunk(pamm_dtype dt) { return dt == PAMM_BF16 ? 8 : 4; }

inline bool dtype_ok(pamm_dtype dt) { return dt == PAMM_F32 || dt == PAMM_BF16; }

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
    int piece_rows;       // P: a generator's rows are cut into pieces of at most P rows
    int64_t nslots;       // upper bound on pieces: floor(b/P) + k
    int col_groups;       // ceil(m / 512): one wave covers 512 columns of a row
    size_t off_perm, off_alpha, off_row0, off_len, off_sbase, off_snum, off_partial, total;
};

inline pamm_status plan_grad(int64_t b, int64_t n, int64_t k, int64_t m, pamm_dtype dt, GradPlan* p) {
    if (!dtype_ok(dt)) return PAMM_ERR_UNSUPPORTED;
    if (b < 1 || n < 1 || m < 1 || k < 1 || b >= (int64_t(1) << 31) || n >= (int64_t(1) << 31) || m >= (int64_t(1) << 31))
        return PAMM_ERR_INVALID_ARG;
    if (k > kMaxGenerators) return PAMM_ERR_UNSUPPORTED;
    if (n % per_chunk(dt) != 0 || m % per_chunk(dt) != 0) return PAMM_ERR_UNSUPPORTED;
    p->col_groups = int((m + 511) / 512);
    // aim at ~2048 single-wave workgroups that carry rows (8 per CU); fewer, longer pieces beyond that
    int64_t want_pieces = (2048 + p->col_groups - 1) / p->col_groups;
    int64_t rows = b / (want_pieces > 0 ? want_pieces : 1);
    int P = 32;
    while (P < 1024 && P * 2 <= rows) P *= 2;
    p->piece_rows = P;
    p->nslots = b / P + k;
    size_t o = 0;
    p->off_perm = o;    o = align_up(o + size_t(b) * 4, 256);
    p->off_alpha = o;   o = align_up(o + size_t(b) * 4, 256);
    p->off_row0 = o;    o = align_up(o + size_t(p->nslots) * 4, 256);
    p->off_len = o;     o = align_up(o + size_t(p->nslots) * 4, 256);
    p->off_sbase = o;   o = align_up(o + size_t(k) * 4, 256);
    p->off_snum = o;    o = align_up(o + size_t(k) * 4, 256);
    p->off_partial = o; o = align_up(o + size_t(p->nslots) * size_t(m) * 4, 256);
    p->total = o;
    return PAMM_OK;
}

}  // namespace pamm
