// Host-only part of libwindq: argument checks, unit geometry, plan layout, effective-bit
// accounting (Eq. 5), workspace sizes.  No kernels here.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "windq_common.hpp"
#include "windq_ws.hpp"

namespace windq {

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int check_matrix(const windq_mat* M) {
    if (M == nullptr || M->data == nullptr) return WINDQ_EINVAL;
    if (M->dtype != WINDQ_F32 && M->dtype != WINDQ_BF16) return WINDQ_EDTYPE;
    if (M->rows <= 0 || M->cols <= 0) return WINDQ_ESHAPE;
    if (M->ld < M->cols || (M->ld % 8) != 0 || (M->cols % 8) != 0) return WINDQ_ESHAPE;
    if (M->rows > (int64_t)1 << 31 || M->ld > (int64_t)1 << 31) return WINDQ_ESHAPE;
    if (!aligned(M->data, 16)) return WINDQ_EINVAL;
    return WINDQ_OK;
}

int make_geometry(const windq_mat* W, int32_t chunk_w, int64_t unit_rows, Geometry* g) {
    const int st = check_matrix(W);
    if (st != WINDQ_OK) return st;
    if (chunk_w < 8 || chunk_w > WINDQ_MAX_CHUNK || (chunk_w % 8) != 0) return WINDQ_ESHAPE;
    if (W->cols % chunk_w != 0) return WINDQ_ESHAPE;
    if (unit_rows < 0) return WINDQ_ESHAPE;
    const int64_t R_u = unit_rows == 0 ? W->rows : unit_rows;
    if (W->rows % R_u != 0) return WINDQ_ESHAPE;
    g->rows = W->rows;
    g->cols = W->cols;
    g->ld = W->ld;
    g->chunk_w = chunk_w;
    g->R_u = R_u;
    g->n_chunks = W->cols / chunk_w;
    g->n_rb = W->rows / R_u;
    g->U = g->n_rb * g->n_chunks;
    g->tiles_per_unit = (R_u + TILE_ROWS - 1) / TILE_ROWS;
    g->n_tiles = g->U * g->tiles_per_unit;
    if (g->n_tiles > (int64_t)0x7fffffff) return WINDQ_ESHAPE;
    return WINDQ_OK;
}

int check_clip_grid(const float* clip_grid, int32_t K) {
    if (clip_grid == nullptr) return WINDQ_EINVAL;
    if (K < 1 || K > WINDQ_MAX_CLIP) return WINDQ_EINVAL;
    for (int32_t k = 0; k < K; ++k) {
        const float p = clip_grid[k];
        if (!(p > 0.0f && p <= 1.0f)) return WINDQ_EINVAL;
        if (k > 0 && !(clip_grid[k] > clip_grid[k - 1])) return WINDQ_EINVAL;
    }
    return WINDQ_OK;
}

int ensure_lds(const void* kernel, size_t bytes) {
    if (bytes <= 64 * 1024) return WINDQ_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
        return WINDQ_EHIP;
    return WINDQ_OK;
}

// Bits x 100 of the seven actions, in the order of Eq. 3.
static const int64_t kCentibits[WINDQ_N_ACTIONS] = {1600, 800, 400, 300, 200, 158, 100};

}  // namespace windq

using namespace windq;

extern "C" {

int64_t windq_bytes_per_group(int32_t action, int32_t chunk_w) {
    if (action < 0 || action >= WINDQ_N_ACTIONS || chunk_w <= 0) return -1;
    if (action == 0) return 0;
    if (action == 5) return ((int64_t)chunk_w + 4) / 5;
    const int64_t bits = kCentibits[action] / 100;
    return ((int64_t)chunk_w * bits + 7) / 8;
}

int windq_plan_layout(const uint8_t* action, int64_t n_units, int64_t rows_per_unit, int32_t chunk_w,
                      int64_t* code_off) {
    if (n_units < 0 || rows_per_unit <= 0 || chunk_w <= 0) return WINDQ_ESHAPE;
    if ((action == nullptr && n_units > 0) || code_off == nullptr) return WINDQ_EINVAL;
    for (int64_t u = 0; u < n_units; ++u)
        if (action[u] >= WINDQ_N_ACTIONS) return WINDQ_EINVAL;
    int64_t pos = 0;
    for (int64_t u = 0; u < n_units; ++u) {
        code_off[u] = pos;
        const int64_t bytes = windq_bytes_per_group(action[u], chunk_w) * rows_per_unit;
        pos += (bytes + 15) / 16 * 16;
    }
    code_off[n_units] = pos;
    return WINDQ_OK;
}

int windq_effective_bits(const uint8_t* action, const int64_t* n_unit, const int64_t* n_prot, int64_t n_units,
                         int64_t* total_centibits, int64_t* total_weights) {
    if (n_units < 0) return WINDQ_ESHAPE;
    if (total_centibits == nullptr || total_weights == nullptr) return WINDQ_EINVAL;
    if (n_units > 0 && (action == nullptr || n_unit == nullptr)) return WINDQ_EINVAL;
    int64_t cb = 0, nw = 0;
    for (int64_t i = 0; i < n_units; ++i) {
        const int a = action[i];
        const int64_t n = n_unit[i];
        const int64_t np = n_prot ? n_prot[i] : 0;
        if (a >= WINDQ_N_ACTIONS || n < 0 || np < 0 || np > n) return WINDQ_EINVAL;
        cb += a == 0 ? 1600 * n : kCentibits[a] * (n - np) + 800 * np;
        nw += n;
    }
    *total_centibits = cb;
    *total_weights = nw;
    return WINDQ_OK;
}

size_t windq_workspace_bytes(int32_t which_call, int32_t dtype, int64_t rows, int64_t cols, int32_t chunk_w,
                             int64_t unit_rows, int32_t K) {
    if (dtype != WINDQ_F32 && dtype != WINDQ_BF16) return 0;
    if (rows <= 0 || cols <= 0) return 0;
    if (which_call == WINDQ_CALL_CALIB_STATS) return calib_ws_bytes(rows, cols);
    windq_mat fake;
    fake.data = reinterpret_cast<const void*>(uintptr_t(256));
    fake.dtype = dtype;
    fake.reserved = 0;
    fake.rows = rows;
    fake.cols = cols;
    fake.ld = cols;
    Geometry g;
    if (make_geometry(&fake, chunk_w, unit_rows, &g) != WINDQ_OK) return 0;
    switch (which_call) {
        case WINDQ_CALL_UNIT_FEATURES: return features_ws_bytes(g, dtype);
        case WINDQ_CALL_FIT_SCORE:
            if (K < 1 || K > WINDQ_MAX_CLIP) return 0;
            return fit_score_ws_bytes(g, K);
        case WINDQ_CALL_APPLY_PLAN: return apply_ws_bytes(g);
        case WINDQ_CALL_SALIENT: return salient_ws_bytes(g);
        case WINDQ_CALL_DEQUANT_GEMV: return dequant_gemv_ws_bytes(g);
        case WINDQ_CALL_UNIT_SALIENCY: return unit_saliency_ws_bytes(g);
        case WINDQ_CALL_DEQUANT: return dequant_ws_bytes(g);
        case WINDQ_CALL_REFINE: return unit_saliency_ws_bytes(g);
        case WINDQ_CALL_FEATURES_FIT_SCORE:
            if (K < 1 || K > WINDQ_MAX_CLIP) return 0;
            return features_ws_bytes(g, dtype) + fit_score_ws_bytes(g, K);
        default: return 0;
    }
}

// Eq. 5 for one unit, in centibits.
static int64_t unit_cost(int a, int64_t n, int64_t n_p) {
    return a == 0 ? 1600 * n : kCentibits[a] * (n - n_p) + 800 * n_p;
}

int windq_heuristic_plan(const float* sal, const int64_t* n_unit, const int64_t* n_prot, int64_t n_units,
                         int64_t target_centibits, uint32_t frac_1bit_ppm, uint32_t frac_ternary_ppm,
                         uint8_t* action, int64_t* total_centibits, int32_t* feasible) {
    if (n_units < 0 || target_centibits < 0 || frac_1bit_ppm > 1000000u || frac_ternary_ppm > 1000000u)
        return WINDQ_EINVAL;
    if (total_centibits == nullptr || feasible == nullptr) return WINDQ_EINVAL;
    if (n_units > 0 && (sal == nullptr || n_unit == nullptr || action == nullptr)) return WINDQ_EINVAL;
    const int64_t U = n_units;
    int64_t total_n = 0;
    for (int64_t u = 0; u < U; ++u) {
        const int64_t np = n_prot != nullptr ? n_prot[u] : 0;
        if (n_unit[u] < 0 || np < 0 || np > n_unit[u] || sal[u] != sal[u]) return WINDQ_EINVAL;
        total_n += n_unit[u];
    }
    // rank: most salient first, equal scores by index
    std::vector<int64_t> order((size_t)U);
    for (int64_t u = 0; u < U; ++u) order[(size_t)u] = u;
    std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) { return sal[a] > sal[b]; });
    auto np_of = [&](int64_t u) { return n_prot != nullptr ? n_prot[u] : (int64_t)0; };
    auto cost = [&](int64_t u, int a) { return unit_cost(a, n_unit[u], np_of(u)); };
    const int64_t n1 = (int64_t)(((unsigned __int128)(uint64_t)U * frac_1bit_ppm) / 1000000u);
    int64_t n158 = (int64_t)(((unsigned __int128)(uint64_t)U * frac_ternary_ppm) / 1000000u);
    if (n158 > U - n1) n158 = U - n1;
    for (int64_t u = 0; u < U; ++u) action[u] = 4;
    for (int64_t i = U - n1; i < U; ++i) action[order[(size_t)i]] = 6;
    for (int64_t i = U - n1 - n158; i < U - n1; ++i) action[order[(size_t)i]] = 5;
    int64_t B = 0;
    for (int64_t u = 0; u < U; ++u) B += cost(u, action[u]);
    const int64_t budget = target_centibits * total_n;
    // over budget: demote one level at a time from the least salient upward
    while (B > budget) {
        bool changed = false;
        for (int64_t i = U - 1; i >= 0; --i) {
            const int64_t u = order[(size_t)i];
            if (action[u] == 4 || action[u] == 5) {
                B += cost(u, action[u] + 1) - cost(u, action[u]);
                action[u] = (uint8_t)(action[u] + 1);
                changed = true;
                if (B <= budget) break;
            }
        }
        if (!changed) break;
    }
    // spend what is left on the most salient units: 2 -> 3 wherever it fits, then 3 -> 4
    const int steps[2][2] = {{4, 3}, {3, 2}};
    for (const auto& st : steps) {
        for (int64_t i = 0; i < U; ++i) {
            const int64_t u = order[(size_t)i];
            if (action[u] == st[0] && B + cost(u, st[1]) - cost(u, st[0]) <= budget) {
                B += cost(u, st[1]) - cost(u, st[0]);
                action[u] = (uint8_t)st[1];
            }
        }
    }
    *total_centibits = B;
    *feasible = B <= budget ? 1 : 0;
    return WINDQ_OK;
}

int windq_fallback_promote(uint8_t* action, const float* err, const float* ref_energy, int64_t n_units,
                           float max_rel_err, int64_t* n_changed) {
    if (n_units < 0 || n_changed == nullptr || !(max_rel_err >= 0.0f)) return WINDQ_EINVAL;
    if (n_units > 0 && (action == nullptr || err == nullptr || ref_energy == nullptr)) return WINDQ_EINVAL;
    for (int64_t u = 0; u < n_units; ++u)
        if (action[u] >= WINDQ_N_ACTIONS) return WINDQ_EINVAL;
    int64_t changed = 0;
    for (int64_t u = 0; u < n_units; ++u) {
        int a = action[u];
        const int a0 = a;
        const double limit = (double)max_rel_err * (double)ref_energy[u];      // exact: two fp32 factors
        while (a != 0 && !((double)err[u * WINDQ_N_ERR + (a - 1)] <= limit)) --a;
        action[u] = (uint8_t)a;
        changed += a != a0 ? 1 : 0;
    }
    *n_changed = changed;
    return WINDQ_OK;
}

const char* windq_status_str(int status) {
    switch (status) {
        case WINDQ_OK: return "ok";
        case WINDQ_EINVAL: return "invalid argument (null or misaligned pointer, bad scalar, bad plan entry)";
        case WINDQ_ESHAPE: return "shape outside the supported limits";
        case WINDQ_EDTYPE: return "unknown dtype";
        case WINDQ_EWORKSPACE: return "workspace missing or too small";
        case WINDQ_EHIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

}  // extern "C"
