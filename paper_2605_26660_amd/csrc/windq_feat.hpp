// What the unit-feature kernels (unit_features.hip) and the tile kernel that makes their first
// pass (fit_score.hip) share: the per-matrix argument block and the launch steps.
#pragma once

#include "windq_common.hpp"
#include "windq_ws.hpp"

namespace windq {

struct FeatArgs {
    const void* W;
    const float* s;
    float* feat;
    double* moments;    // [n_tiles][4][4]
    uint32_t* above;    // fp32 inputs
    uint32_t* hist;     // [U][FEAT_BINS] (bf16), [3][U][FEAT_BINS] (fp32)
    uint32_t* fine;     // bf16 inputs: [n_tiles][FEAT_WIN][8] full-resolution counts around each tile's bulk
    uint32_t* anchor;   //              [n_tiles] last bin of that record; << 16, bin of the tile's largest key
    uint32_t* list_count;   //          units whose P99 the tiles' records do not decide ...
    uint32_t* list;     //              ... [U] their indices, in no particular order
    uint32_t sparse_key;    //          smallest bf16 key whose value is >= 1e-6
    Geometry g;
    int64_t bpu;        // workgroups per unit (passes after the first)
    int64_t mparts;     // moment records per unit
    float sparse_thr;   // smallest fp32 that is >= 1e-6: (|w| < 1e-6) == (|w| < sparse_thr) for fp32 |w|
    uint64_t rank;      // ceil(0.99 n), 1-based
};

// A launch covers up to WINDQ_MAX_BATCH matrices (one chunk width, one element type): the
// workgroups of the pass kernels, the units of the finish kernel and the counters the init
// kernel clears are numbered one matrix after the other.
struct FeatBatch {
    int32_t n;
    int32_t dtype;
    int64_t block_start[WINDQ_MAX_BATCH + 1];
    int64_t unit_start[WINDQ_MAX_BATCH + 1];
    int64_t init_start[WINDQ_MAX_BATCH + 1];     // in workgroups of 256 counters
    int64_t blocks_total, units_total, init_total;
    FeatArgs m[WINDQ_MAX_BATCH];
};

// One matrix as the feature launch steps see it.
struct FeatItem {
    const windq_mat* W;
    const float* s;
    float* feat;
    void* ws;           // features layout at its start
    size_t ws_bytes;
};

// Checks every item and fills B; nothing is launched.  (unit_features.hip)
int features_fill(const FeatItem* items, int32_t n, int32_t chunk_w, int64_t unit_rows, FeatBatch* B);
// Clears the histograms.  (unit_features.hip)
int features_launch_init(const FeatBatch& B, hipStream_t hs);
// The first pass by itself: per tile, moments, counts and the first-digit histogram.  (fit_score.hip)
int features_launch_tiles(const FeatBatch& B, hipStream_t hs);
// Everything after the first pass: bf16, the finish kernel (with the exact pass over the units it lists);
// fp32, the refining passes and the finish kernel.  (unit_features.hip)
int features_launch_rest(const FeatBatch& B, hipStream_t hs);

}  // namespace windq
