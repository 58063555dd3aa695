// windq_refine_plan: windq_apply_plan with refined scales.  The paper fits each operator's
// scale by a short local optimisation of the reconstruction loss on the unit (App. "Per-unit
// Scale Optimization": ~10 optimiser steps, no model-wide backward pass).  The deterministic
// stand-in here: every group is seeded with its grid fit, then alternates
//     assign codes by the normative fp32 steps  |  solve the activation-weighted
//     least-squares problem for the group's parameters in closed form
// for n_iter rounds; neither half-step can raise the loss.  Uniform: minimise
// sum a_c (w - lo - q step)^2 over (lo, step) by the 2x2 normal equations; ternary:
// gamma = sum a q w / sum a q^2; binary (signs fixed): alpha = sum a |w| / sum a.
// The sums are fp64 in column order from plain multiplies and adds (this file is compiled
// with contraction off), the parameters are rounded to fp32 after every solve: the results
// are defined to the bit, so codes and stored parameters can be checked exactly.
//
// One wavefront per 64-row tile, one lane per group, tile in LDS (as the general apply-plan
// kernel): a group's refinement is a lane-private sequence.  fp64 arithmetic at ~15 operations
// per weight and round: bound by the fp64 ALU, not by HBM; it runs once per chosen plan.
#include <float.h>

#include "windq_common.hpp"
#include "windq_group.hpp"
#include "windq_ws.hpp"

namespace windq {

struct RefineArgs {
    const void* W;
    const float* s;
    const uint8_t* mask;       // or null
    int64_t mask_ld;
    const uint8_t* action;
    const uint8_t* clip_idx;   // or null
    const int64_t* code_off;
    uint8_t* codes;
    int64_t codes_bytes;
    float* scale;
    float* offset;
    double* part;              // [n_tiles]
    float* err;                // [U]
    Geometry g;
};

// A launch covers up to WINDQ_MAX_BATCH matrices (one chunk width, one element type, one clip
// grid and round count): their tiles and units are numbered one matrix after the other.
struct RefineBatch {
    int32_t n;
    int32_t K;
    int32_t n_iter;
    int64_t tile_start[WINDQ_MAX_BATCH + 1];
    int64_t unit_start[WINDQ_MAX_BATCH + 1];
    RefineArgs m[WINDQ_MAX_BATCH];
    ClipGrid grid;
};

__device__ __forceinline__ bool kept_bit(uint32_t m, int j) { return ((m >> j) & 1u) == 0u; }

// The sums of one round of the uniform refinement over a group.  S0 = sum a and T0 = sum a w do
// not depend on the codes: the first round computes them (FIRST), later rounds reuse them; the
// order of every sum is the column order either way.
template <int DT, bool FIRST>
__device__ __forceinline__ void uniform_sums(const char* wrow, const uint8_t* mrow, const double* acol, int32_t G,
                                             float lo, float inv, float qmax, double* S0_io, double* T0_io,
                                             double* S1_o, double* S2_o, double* T1_o) {
    double S0 = 0.0, S1 = 0.0, S2 = 0.0, T0 = 0.0, T1 = 0.0;
    for (int32_t c = 0; c < G; c += 8) {
        float w[8];
        read8<DT>(wrow, c, w);
        const uint32_t m = mrow != nullptr ? mrow[c >> 3] : 0u;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float u = w[j] - lo;
            const float t = u * inv;
            const double q = (double)__builtin_amdgcn_fmed3f(__builtin_rintf(t), 0.0f, qmax);
            const double a = kept_bit(m, j) ? acol[c + j] : 0.0;      // a masked weight adds zeros
            const double wd = (double)w[j];
            const double aq = a * q;
            if (FIRST) {
                S0 = S0 + a;
                T0 = T0 + a * wd;
            }
            S1 = S1 + aq;
            S2 = S2 + aq * q;
            T1 = T1 + aq * wd;
        }
    }
    if (FIRST) {
        *S0_io = S0;
        *T0_io = T0;
    }
    *S1_o = S1;
    *S2_o = S2;
    *T1_o = T1;
}

template <int DT>
__device__ __forceinline__ void refine_uniform(const char* wrow, const uint8_t* mrow, const double* acol,
                                               int32_t G, float qmax, int n_iter, float* lo_io, float* d_io) {
    float lo = *lo_io, d = *d_io;
    double S0 = 0.0, T0 = 0.0;
    for (int it = 0; it < n_iter; ++it) {
        if (!(d >= FLT_MIN)) break;
        const float inv = 1.0f / d;
        double S1, S2, T1;
        if (it == 0) uniform_sums<DT, true>(wrow, mrow, acol, G, lo, inv, qmax, &S0, &T0, &S1, &S2, &T1);
        else uniform_sums<DT, false>(wrow, mrow, acol, G, lo, inv, qmax, &S0, &T0, &S1, &S2, &T1);
        const double det = S0 * S2 - S1 * S1;
        if (!(det > 0.0)) break;
        const double d_new = (S0 * T1 - S1 * T0) / det;
        const double lo_new = (T0 - S1 * d_new) / S0;
        const float d32 = (float)d_new, lo32 = (float)lo_new;
        if (!(d32 >= FLT_MIN)) break;
        lo = lo32;
        d = d32;
    }
    *lo_io = lo;
    *d_io = d;
}

template <int DT>
__device__ __forceinline__ float refine_ternary(const char* wrow, const uint8_t* mrow, const double* acol,
                                                int32_t G, int n_iter, float gamma) {
    for (int it = 0; it < n_iter; ++it) {
        if (!(gamma >= FLT_MIN)) break;
        const float inv = 1.0f / gamma;
        double N1 = 0.0, D1 = 0.0;
        for (int32_t c = 0; c < G; c += 8) {
            float w[8];
            read8<DT>(wrow, c, w);
            const uint32_t m = mrow != nullptr ? mrow[c >> 3] : 0u;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float t = w[j] * inv;
                const double q = (double)__builtin_amdgcn_fmed3f(__builtin_rintf(t), -1.0f, 1.0f);
                const double a = kept_bit(m, j) ? acol[c + j] : 0.0;
                const double aq = a * q;
                N1 = N1 + aq * (double)w[j];
                D1 = D1 + aq * q;
            }
        }
        if (!(D1 > 0.0)) break;
        const float g = (float)(N1 / D1);
        if (!(g >= FLT_MIN)) break;
        gamma = g;
    }
    return gamma;
}

template <int DT>
__device__ __forceinline__ float refine_binary(const char* wrow, const uint8_t* mrow, const double* acol,
                                               int32_t G, float alpha) {
    double N1 = 0.0, D1 = 0.0;
    for (int32_t c = 0; c < G; c += 8) {
        float w[8];
        read8<DT>(wrow, c, w);
        const uint32_t m = mrow != nullptr ? mrow[c >> 3] : 0u;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const double a = kept_bit(m, j) ? acol[c + j] : 0.0;
            N1 = N1 + a * (double)fabsf(w[j]);
            D1 = D1 + a;
        }
    }
    return D1 > 0.0 ? (float)(N1 / D1) : alpha;
}

// Activation-weighted error of a group under its final parameters (fp64; w_hat from the
// stored fp32 numbers, as everywhere).
template <int DT>
__device__ __forceinline__ double group_error(const char* wrow, const uint8_t* mrow, const double* acol,
                                              int32_t G, int a, float sc, float of) {
    const int bits = a == 1 ? 8 : (a == 2 ? 4 : (a == 3 ? 3 : 2));
    const float qmax = (float)((1 << bits) - 1);
    const float inv = sc >= FLT_MIN ? 1.0f / sc : 0.0f;
    double e = 0.0;
    for (int32_t c = 0; c < G; c += 8) {
        float w[8];
        read8<DT>(wrow, c, w);
        const uint32_t m = mrow != nullptr ? mrow[c >> 3] : 0u;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            double what;
            if (a <= 4) {
                const float t = (w[j] - of) * inv;
                what = (double)of + (double)__builtin_amdgcn_fmed3f(__builtin_rintf(t), 0.0f, qmax) * (double)sc;
            } else if (a == 5) {
                what = (double)sc * (double)__builtin_amdgcn_fmed3f(__builtin_rintf(w[j] * inv), -1.0f, 1.0f);
            } else {
                what = w[j] >= 0.0f ? (double)sc : -(double)sc;
            }
            const double d = (double)w[j] - what;
            const double ac = kept_bit(m, j) ? acol[c + j] : 0.0;
            e = e + ac * d * d;
        }
    }
    return e;
}

constexpr int RF_THREADS = 64;

template <int DT>
__global__ __launch_bounds__(RF_THREADS) void refine_plan_kernel(const RefineBatch B) {
    extern __shared__ char smem[];
    const int mi = batch_index(B.tile_start, B.n, blockIdx.x);
    const RefineArgs& A = B.m[mi];
    const TileCoord tc = tile_coord(A.g, (int64_t)blockIdx.x - B.tile_start[mi]);
    const int32_t G = A.g.chunk_w;
    const int32_t row_bytes = G * Elem<DT>::bytes + 16;
    char* tile = smem;
    double* acol = reinterpret_cast<double*>(smem + TILE_ROWS * row_bytes);     // s_c^2 of the chunk's columns
    const int32_t mstride = mask_row_stride(G);
    uint8_t* mtile = reinterpret_cast<uint8_t*>(acol + G);                       // the tile's mask bytes (masked calls)
    const int lane = threadIdx.x;
    const bool valid = lane < tc.nrows;
    const int64_t gidx = tc.u * A.g.R_u + tc.lrow0 + lane;
    const size_t tile_idx = (size_t)tc.u * (size_t)A.g.tiles_per_unit + (size_t)tc.t;

    int a = A.action[tc.u];
    if (a >= WINDQ_N_ACTIONS) a = 0;
    const int64_t bpg = dev_bytes_per_group(a, G);
    const int64_t base = A.code_off[tc.u];
    const int64_t payload = bpg * A.g.R_u;
    const int64_t padded = (payload + 15) & ~(int64_t)15;
    if (base < 0 || (base & 15) != 0 || base + padded > A.codes_bytes) a = 0;
    if (a == 0) {
        if (valid) {
            A.scale[gidx] = 0.0f;
            A.offset[gidx] = 0.0f;
        }
        if (lane == 0) A.part[tile_idx] = 0.0;
        return;
    }

    load_tile_raw<DT>(A.W, A.g.ld, tc, G, tile);
    for (int32_t c = lane; c < G; c += RF_THREADS) {
        const double sv = (double)A.s[tc.col0 + c];
        acol[c] = sv * sv;
    }
    if (A.mask != nullptr) load_mask_tile(A.mask, A.mask_ld, tc, G, mtile);
    __syncthreads();

    char* wrow = tile + lane * row_bytes;
    double err = 0.0;
    if (valid) {
        const uint8_t* mrow = A.mask != nullptr ? mtile + lane * mstride : nullptr;
        uint8_t* dst = reinterpret_cast<uint8_t*>(wrow);
        float sc = 0.0f, of = 0.0f;
        if (a <= 4) {
            float p = 1.0f;
            if (A.clip_idx != nullptr) {
                int k = A.clip_idx[tc.u * 4 + (a - 1)];
                k = k < B.K ? k : B.K - 1;
                p = B.grid.p[k];
            }
            const int bits = a == 1 ? 8 : (a == 2 ? 4 : (a == 3 ? 3 : 2));
            const float qmax = (float)((1 << bits) - 1);
            float mn, mx;
            group_min_max<DT>(wrow, mrow, G, &mn, &mx);
            uniform_params(mn, mx, p, qmax, &of, &sc);
            refine_uniform<DT>(wrow, mrow, acol, G, qmax, B.n_iter, &of, &sc);
            err = group_error<DT>(wrow, mrow, acol, G, a, sc, of);
            switch (a) {
                case 1: uniform_pack<DT, 8>(wrow, mrow, G, of, sc, dst); break;
                case 2: uniform_pack<DT, 4>(wrow, mrow, G, of, sc, dst); break;
                case 3: uniform_pack<DT, 3>(wrow, mrow, G, of, sc, dst); break;
                default: uniform_pack<DT, 2>(wrow, mrow, G, of, sc, dst); break;
            }
        } else if (a == 5) {
            sc = group_abs_mean<DT>(wrow, mrow, G);
            sc = sc >= FLT_MIN ? sc : 0.0f;
            sc = refine_ternary<DT>(wrow, mrow, acol, G, B.n_iter, sc);
            err = group_error<DT>(wrow, mrow, acol, G, a, sc, 0.0f);
            ternary_pack<DT>(wrow, mrow, G, sc, dst);
        } else {
            sc = group_abs_mean<DT>(wrow, mrow, G);
            if (B.n_iter > 0) sc = refine_binary<DT>(wrow, mrow, acol, G, sc);
            err = group_error<DT>(wrow, mrow, acol, G, a, sc, 0.0f);
            binary_pack<DT>(wrow, mrow, G, dst);
        }
        A.scale[gidx] = sc;
        A.offset[gidx] = of;
    }
    // rows of the tile in order (lane 0 first): a fixed-order fp64 sum
    err = wave_sum(err);
    if (lane == 0) A.part[tile_idx] = err;
    __syncthreads();
    copy_out_rows(tile, row_bytes, (int32_t)bpg, tc.nrows, A.codes + base + tc.lrow0 * bpg, lane, RF_THREADS);
    if (padded != payload && tc.t == A.g.tiles_per_unit - 1 && lane < padded - payload)
        A.codes[base + payload + lane] = 0;
}

// err[u] = the sum of unit u's tile partials; one workgroup per unit.
__global__ __launch_bounds__(256) void refine_finalize_kernel(const RefineBatch B) {
    __shared__ double red[4];
    const int mi = batch_index(B.unit_start, B.n, blockIdx.x);
    const RefineArgs& A = B.m[mi];
    const int64_t u = (int64_t)blockIdx.x - B.unit_start[mi];
    const double t = unit_partial_sum<256>(A.part + (size_t)u * (size_t)A.g.tiles_per_unit, A.g.tiles_per_unit, red);
    if (threadIdx.x == 0) A.err[u] = (float)t;
}

}  // namespace windq

using namespace windq;

static int refine_launch(const windq_refine_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows,
                         const float* clip_grid, int32_t K, int32_t n_iter, void* stream) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    if (n_iter < 0 || n_iter > 64) return WINDQ_EINVAL;
    bool any_idx = false, any_mask = false;
    for (int32_t i = 0; i < n; ++i) {
        any_idx = any_idx || items[i].clip_idx != nullptr;
        any_mask = any_mask || items[i].mask != nullptr;
    }
    int st;
    if (any_idx || clip_grid != nullptr) {
        st = check_clip_grid(clip_grid, K);
        if (st != WINDQ_OK) return st;
    } else {
        K = 1;
    }
    RefineBatch B;
    B.n = n;
    B.K = K;
    B.n_iter = n_iter;
    for (int k = 0; k < WINDQ_MAX_CLIP; ++k) B.grid.p[k] = clip_grid != nullptr ? clip_grid[k < K ? k : K - 1] : 1.0f;
    int64_t tiles = 0, units = 0;
    for (int32_t i = 0; i < n; ++i) {
        const windq_refine_item& it = items[i];
        RefineArgs& A = B.m[i];
        if (it.W == nullptr) return WINDQ_EINVAL;
        st = make_geometry(it.W, chunk_w, unit_rows, &A.g);
        if (st != WINDQ_OK) return st;
        if (it.s == nullptr || it.action == nullptr || it.code_off == nullptr || it.scale == nullptr ||
            it.offset == nullptr || it.err == nullptr)
            return WINDQ_EINVAL;
        if (it.codes == nullptr && it.codes_bytes != 0) return WINDQ_EINVAL;
        if (it.codes != nullptr && !aligned(it.codes, 16)) return WINDQ_EINVAL;
        if (!aligned(it.code_off, 8)) return WINDQ_EINVAL;
        if (it.W->dtype != items[0].W->dtype) return WINDQ_EINVAL;      // one kernel per launch
        if (it.ws == nullptr || it.ws_bytes < unit_saliency_ws_bytes(A.g) || !aligned(it.ws, 256)) return WINDQ_EWORKSPACE;
        A.W = it.W->data;
        A.s = it.s;
        A.mask = it.mask;
        A.mask_ld = it.W->cols / 8;
        A.action = it.action;
        A.clip_idx = clip_grid != nullptr ? it.clip_idx : nullptr;
        A.code_off = it.code_off;
        A.codes = it.codes;
        A.codes_bytes = (int64_t)it.codes_bytes;
        A.scale = it.scale;
        A.offset = it.offset;
        A.part = static_cast<double*>(it.ws);
        A.err = it.err;
        B.tile_start[i] = tiles;
        B.unit_start[i] = units;
        tiles += A.g.n_tiles;
        units += A.g.U;
    }
    for (int32_t i = n; i <= WINDQ_MAX_BATCH; ++i) {
        B.tile_start[i] = tiles;
        B.unit_start[i] = units;
    }
    for (int32_t i = n; i < WINDQ_MAX_BATCH; ++i) B.m[i] = B.m[0];
    if (tiles > (int64_t)0x7fffffff) return WINDQ_ESHAPE;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int32_t dtype = items[0].W->dtype;
    const size_t lds = raw_tile_lds_bytes(dtype, chunk_w) + (size_t)chunk_w * sizeof(double) +
                       (any_mask ? mask_tile_lds_bytes(chunk_w) : 0);
    const dim3 grid((unsigned)tiles);
    if (dtype == WINDQ_BF16) {
        st = ensure_lds(reinterpret_cast<const void*>(&refine_plan_kernel<WINDQ_BF16>), lds);
        if (st != WINDQ_OK) return st;
        hipLaunchKernelGGL(refine_plan_kernel<WINDQ_BF16>, grid, dim3(RF_THREADS), lds, hs, B);
    } else {
        st = ensure_lds(reinterpret_cast<const void*>(&refine_plan_kernel<WINDQ_F32>), lds);
        if (st != WINDQ_OK) return st;
        hipLaunchKernelGGL(refine_plan_kernel<WINDQ_F32>, grid, dim3(RF_THREADS), lds, hs, B);
    }
    hipLaunchKernelGGL(refine_finalize_kernel, dim3((unsigned)units), dim3(256), 0, hs, B);
    return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
}

extern "C" int windq_refine_plan(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows,
                                 const uint8_t* mask, const uint8_t* action, const uint8_t* clip_idx,
                                 const float* clip_grid, int32_t K, int32_t n_iter, const int64_t* code_off,
                                 uint8_t* codes, size_t codes_bytes, float* scale, float* offset, float* err, void* ws,
                                 size_t ws_bytes, void* stream) {
    const windq_refine_item it = {W, s, mask, action, clip_idx, code_off, codes, codes_bytes, scale, offset, err, ws, ws_bytes};
    return refine_launch(&it, 1, chunk_w, unit_rows, clip_grid, K, n_iter, stream);
}

extern "C" int windq_refine_plan_batch(const windq_refine_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows,
                                       const float* clip_grid, int32_t K, int32_t n_iter, void* stream) {
    return refine_launch(items, n, chunk_w, unit_rows, clip_grid, K, n_iter, stream);
}
