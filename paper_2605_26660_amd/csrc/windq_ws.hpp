// Workspace layouts: one place that both windq_workspace_bytes and the launchers use.
#pragma once

#include "windq_common.hpp"

namespace windq {

// ---- calib_stats: per slab of CALIB_SLAB_ROWS tokens, per channel, two fp64 partial sums
constexpr int CALIB_SLAB_ROWS = 32;
inline int64_t calib_slabs(int64_t rows) { return (rows + CALIB_SLAB_ROWS - 1) / CALIB_SLAB_ROWS; }
inline size_t calib_ws_bytes(int64_t rows, int64_t cols) {
    return round_up((size_t)calib_slabs(rows) * (size_t)cols * 2 * sizeof(double), 256);
}

// ---- fit_score: per tile, one fp64 partial per candidate, then the list of units whose 8-bit
// candidate is scored again on the exact route
// candidates: [b][k] for b in 8,4,3,2 (index b*K + k); then for each quarter of the chunk's
// columns: ternary, binary, reference energy (12 slots); then [k] the variance term of the
// 8-bit short route's rounding noise at clip index k
__host__ __device__ inline int32_t fit_score_ncand(int32_t K) { return 5 * K + 12; }
__host__ __device__ inline int32_t fit_score_noise_slot(int32_t K) { return 4 * K + 12; }
// What fit+score prepares once per chunk of columns (it depends on s alone): the activation scales
// of the columns that take the short 8-bit route (0 for the others), the list of the others, their
// number (-1: every column takes the exact route) and sum s_c^4 / sum s_c^2 over the short route.
constexpr int FS_HMAX = WINDQ_MAX_CHUNK / 8;   // most columns a chunk may send down the exact 8-bit route on their own
inline __host__ __device__ int32_t colsel_words(int32_t chunk_w) { return chunk_w + FS_HMAX + 4; }   // 4-byte words per chunk

struct FitScoreLayout {
    size_t partial;      // [n_tiles][ncand] fp64
    size_t redo_count;   // u32: units on the list
    size_t redo_list;    // [U] u32
    size_t colsel;       // [n_chunks][colsel_words] the chunks' column selection
    size_t total;
};
inline FitScoreLayout fit_score_layout(const Geometry& g, int32_t K) {
    FitScoreLayout L;
    size_t pos = 0;
    L.partial = pos;     pos = round_up(pos + (size_t)g.n_tiles * (size_t)fit_score_ncand(K) * sizeof(double), 256);
    L.redo_count = pos;  pos += 256;
    L.redo_list = pos;   pos = round_up(pos + (size_t)g.U * sizeof(uint32_t), 256);
    L.colsel = pos;      pos = round_up(pos + (size_t)g.n_chunks * (size_t)colsel_words(g.chunk_w) * 4, 256);
    L.total = pos;
    return L;
}
inline size_t fit_score_ws_bytes(const Geometry& g, int32_t K) { return fit_score_layout(g, K).total; }

// ---- unit_features
// The first pass (moments, counts, histograms) works tile by tile, each of the four wavefronts of a
// workgroup on a quarter of the chunk's columns.
//   moments  [n_tiles][4][4] fp64   per (tile, column quarter): sum w, sum w^2, sum |w|, count(|w| < 1e-6)
// bf16 inputs (15-bit keys = the magnitude bits; first radix digit = key >> 4, 2048 bins):
//   hist     [U][FEAT_BINS] u32     histogram of the first digit; keys below / above the range the tile
//                                   kernel resolves are lumped into its first / last bin
//   fine     [n_tiles][FEAT_WIN][8] u32   per tile, the full-resolution counts (two 16-bit counters per
//                                   dword: even key low, odd key high) of FEAT_WIN first-digit bins
//                                   around the tile's bulk
//   anchor   [n_tiles] u32          the last of those bins; << 16, the bin of the tile's largest key
//   list_count u32, list [U] u32    units whose P99 the records do not decide
// fp32 inputs (31-bit keys, digits 11 + 11 + 9): the later passes cover FEAT_TPB consecutive tiles of one
// unit per workgroup ("block" below)
//   above    [n_blocks]    u32    count(|w| > 0.5 P99)
//   hist     [3][U][FEAT_BINS] u32  histogram of radix digit 0, 1, 2
constexpr int FEAT_DIGIT_BITS = 11;
constexpr int FEAT_BINS = 1 << FEAT_DIGIT_BITS;
constexpr int FEAT_TPB = 2;
constexpr int FEAT_QUARTERS = 4;
// bf16: the tile kernel's LDS histogram resolves FEAT_FINE_NCOARSE first-digit bins key by key,
// 2^-21.1 <= |w| < 13.5 between its two lumping end bins (8 dwords of two counters per first-digit bin).
constexpr int FEAT_FINE_COARSE0 = 847;
constexpr int FEAT_FINE_NCOARSE = 200;
constexpr int FEAT_FINE_PAIRS = FEAT_FINE_NCOARSE * 8;
constexpr int FEAT_WIN = 64;
struct FeatLayout {
    int64_t bpu;       // workgroups per unit (later passes, fp32)
    int64_t n_blocks;
    int64_t mparts;    // moment records per unit: tiles x column quarters
    size_t moments, above, hist, fine, anchor, list_count, list, total;
};
inline FeatLayout features_layout(const Geometry& g, int32_t dtype) {
    FeatLayout L;
    L.bpu = (g.tiles_per_unit + FEAT_TPB - 1) / FEAT_TPB;
    L.n_blocks = g.U * L.bpu;
    L.mparts = g.tiles_per_unit * FEAT_QUARTERS;
    size_t pos = 0;
    L.moments = pos; pos = round_up(pos + (size_t)g.n_tiles * FEAT_QUARTERS * 4 * sizeof(double), 256);
    L.above = L.fine = L.anchor = L.list_count = L.list = 0;
    if (dtype == WINDQ_BF16) {
        L.hist = pos;       pos = round_up(pos + (size_t)g.U * FEAT_BINS * sizeof(uint32_t), 256);
        L.list_count = pos; pos += 256;
        L.list = pos;       pos = round_up(pos + (size_t)g.U * sizeof(uint32_t), 256);
        L.anchor = pos;     pos = round_up(pos + (size_t)g.n_tiles * sizeof(uint32_t), 256);
        L.fine = pos;       pos = round_up(pos + (size_t)g.n_tiles * FEAT_WIN * 8 * sizeof(uint32_t), 256);
    } else {
        L.above = pos;   pos = round_up(pos + (size_t)L.n_blocks * sizeof(uint32_t), 256);
        L.hist = pos;    pos = round_up(pos + (size_t)3 * g.U * FEAT_BINS * sizeof(uint32_t), 256);
    }
    L.total = pos;
    return L;
}
inline size_t features_ws_bytes(const Geometry& g, int32_t dtype) { return features_layout(g, dtype).total; }

// ---- salient-weight protection (select and encode share one layout)
//   hist      [3][U][FEAT_BINS] u32   histograms of the three saliency-key digits
//   prefix, rank, need  [U] u32       selection state per unit
//   flag      [U] u32                 1: the unit's threshold bin holds more keys than its candidate list
//   n_flagged u32, flagged [U] u32    those units
//   cand_count [U] u32, cand [U][cap] (key, position) u32 pairs: the keys of the threshold's first-digit bin
//   cnt       [n_tiles] u32           keys equal to the threshold per tile (flagged units with split ties)
//   eq_before [n_tiles] u32           ties in earlier tiles of the unit
//   tile_max  [n_tiles] f32           largest protected magnitude per tile
//   row_off   [U * R_u] u32           protected weights in earlier rows of the unit
//   err_part  [n_tiles] f64           INT8 error per tile
struct SalientLayout {
    size_t hist, prefix, rank, need, flag, n_flagged, flagged, cand_count, cand, cnt, eq_before, tile_max, row_off, err_part, total;
    uint32_t cap;      // candidates a unit can list
};
// A thirty-second of the unit's weights, at least 256 (a first-digit bin is an eighth of an octave:
// around the 97th-99.5th percentile of the saliencies it holds well under 1 % of a unit).
inline uint32_t salient_cand_cap(const Geometry& g) {
    const uint64_t n = (uint64_t)g.R_u * (uint64_t)g.chunk_w;
    uint64_t c = n / 32;
    if (c < 256) c = 256;
    if (c > n) c = n;
    return (uint32_t)c;
}
inline SalientLayout salient_layout(const Geometry& g) {
    SalientLayout L;
    L.cap = salient_cand_cap(g);
    size_t pos = 0;
    L.hist = pos;      pos = round_up(pos + (size_t)3 * g.U * FEAT_BINS * sizeof(uint32_t), 256);
    L.prefix = pos;    pos = round_up(pos + (size_t)g.U * sizeof(uint32_t), 256);
    L.rank = pos;      pos = round_up(pos + (size_t)g.U * sizeof(uint32_t), 256);
    L.need = pos;      pos = round_up(pos + (size_t)g.U * sizeof(uint32_t), 256);
    L.flag = pos;      pos = round_up(pos + (size_t)g.U * sizeof(uint32_t), 256);
    L.n_flagged = pos; pos += 256;
    L.flagged = pos;   pos = round_up(pos + (size_t)g.U * sizeof(uint32_t), 256);
    L.cand_count = pos; pos = round_up(pos + (size_t)g.U * sizeof(uint32_t), 256);
    L.cand = pos;      pos = round_up(pos + (size_t)g.U * (size_t)L.cap * 2 * sizeof(uint32_t), 256);
    L.cnt = pos;       pos = round_up(pos + (size_t)g.n_tiles * sizeof(uint32_t), 256);
    L.eq_before = pos; pos = round_up(pos + (size_t)g.n_tiles * sizeof(uint32_t), 256);
    L.tile_max = pos;  pos = round_up(pos + (size_t)g.n_tiles * sizeof(float), 256);
    L.row_off = pos;   pos = round_up(pos + (size_t)g.U * (size_t)g.R_u * sizeof(uint32_t), 256);
    L.err_part = pos;  pos = round_up(pos + (size_t)g.n_tiles * sizeof(double), 256);
    L.total = pos;
    return L;
}
inline size_t salient_ws_bytes(const Geometry& g) { return salient_layout(g).total; }

// ---- unit saliency: one fp64 partial per tile
inline size_t unit_saliency_ws_bytes(const Geometry& g) { return round_up((size_t)g.n_tiles * sizeof(double), 256); }

// ---- dequant: one fp64 partial per (tile, row pass); a pass is the rows 256 threads cover at
// eight columns per lane, so a 64-row tile has chunk_w / 32 of them (at least one)
__host__ __device__ inline int32_t dequant_passes(int32_t chunk_w) { return chunk_w >= 32 ? chunk_w / 32 : 1; }
inline size_t dequant_ws_bytes(const Geometry& g) {
    return round_up((size_t)g.n_tiles * (size_t)dequant_passes(g.chunk_w) * sizeof(double), 256);
}

// ---- the product from the artefact: one fp64 partial per (row, chunk)
inline size_t dequant_gemv_ws_bytes(const Geometry& g) {
    return round_up((size_t)g.rows * (size_t)g.n_chunks * sizeof(double), 256);
}

// ---- apply_plan needs no scratch; a token size keeps "ws != NULL" uniform across calls
inline size_t apply_ws_bytes(const Geometry&) { return 256; }

}  // namespace windq
