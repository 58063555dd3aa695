// windq_fit_score_all_bits: fit the lightweight quantizer of every unit at all six
// bit-widths and score each fit by the activation-aware reconstruction error
// (Sec. 3.5 "Quantization Engine and Bit Accounting"; App. "Per-unit Scale
// Optimization": per-group scales, group size = chunk size).
//
// Work per weight: 4 bit-widths x K clip ratios + ternary + binary = 4K+2 candidate
// quantizers, about 23 vector instructions per (weight, clip ratio).  At K = 20 that
// is ~480 instructions per 2-byte weight: the kernel is bound by the vector ALU, not by
// HBM, by a factor of ~40.  The design therefore minimises instructions per candidate:
//   * lane-per-group (see windq_common.hpp): quantizer parameters are lane-private, so
//     each is computed exactly once; the activation weight a_c = s_c^2 is wave-uniform
//     and arrives by scalar loads;
//   * all arithmetic in the inner loop is fp64.  On gfx950 fp64 FMA/ADD/MUL issue at
//     the same rate as (unpacked) fp32, so exactness is free: residuals w - w_hat are
//     formed without cancellation error and the unit errors agree with an fp64
//     reference to ~1e-12;
//   * rounding to the nearest code is one FMA that adds 1.5*2^52 to t = (w-lo)/step and
//     one subtract; the clamp to the code range is done once per clip ratio on (w-lo),
//     shared by the four bit-widths (clamping (w-lo) to [0, hi-lo] before rounding
//     yields the same code as clamping the rounded code to [0, 2^b-1]);
//   * the four wavefronts of a workgroup share the LDS tile and split the clip grid.
// Rounding decisions are taken on the fp64 product here, on the fp32 product in
// windq_apply_plan; where they differ the weight sits within 1e-7 steps of a rounding
// boundary, where both codes give the same squared error to within 1e-6 of itself.
#include <float.h>

#include "windq_common.hpp"
#include "windq_ws.hpp"

namespace windq {

constexpr int FS_THREADS = 256;
constexpr int FS_WAVES = FS_THREADS / 64;
constexpr int FS_KB = 5;   // clip ratios evaluated together by one wavefront pass
constexpr double RNE_MAGIC = 6755399441055744.0;   // 1.5 * 2^52: x + M - M rounds x to nearest-even integer

struct FitScoreArgs {
    const void* W;
    const float* s;
    double* partial;   // [n_tiles][4K+3]
    Geometry g;
    int32_t K;
    int32_t n_kpass;   // ceil(K / FS_KB)
    ClipGrid grid;
};

// One weight against FS_KB clip ratios x 4 bit-widths.
__device__ __forceinline__ void score_weight(const double w, const double a, const double (&lo)[FS_KB],
                                             const double (&rg)[FS_KB], const double (&inv)[FS_KB][4],
                                             const double (&dl)[FS_KB][4], double (&acc)[FS_KB][4]) {
#pragma unroll
    for (int i = 0; i < FS_KB; ++i) {
        const double u = w - lo[i];
        const double uc = fmin(fmax(u, 0.0), rg[i]);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const double q = fma(uc, inv[i][b], RNE_MAGIC) - RNE_MAGIC;   // nearest code, already in range
            const double r = fma(-q, dl[i][b], u);                        // w - (lo + q*step)
            acc[i][b] = fma(a * r, r, acc[i][b]);
        }
    }
}

template <int DT>
__global__ __launch_bounds__(FS_THREADS) void fit_score_kernel(const FitScoreArgs A) {
    extern __shared__ float tile[];
    const TileCoord tc = tile_coord(A.g, blockIdx.x);
    const int32_t G = A.g.chunk_w;
    load_tile<DT>(A.W, A.g.ld, tc, G, tile);
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const bool valid = lane < tc.nrows;
    const float* __restrict__ wrow = tile + lane * (G + LDS_PAD);
    const float* __restrict__ s_chunk = A.s + tc.col0;
    const int32_t K = A.K;
    double* __restrict__ out = A.partial + ((size_t)tc.u * (size_t)A.g.tiles_per_unit + (size_t)tc.t) *
                                               (size_t)fit_score_ncand(K);

    // Group statistics: min, max, S1 = sum |w| in fp64 in column order (exact for bf16).
    float mn = wrow[0], mx = wrow[0];
    double S1 = 0.0;
    for (int32_t c = 0; c < G; c += 4) {
        const float4 v = *reinterpret_cast<const float4*>(wrow + c);
        mn = fminf(fminf(mn, v.x), fminf(v.y, fminf(v.z, v.w)));
        mx = fmaxf(fmaxf(mx, v.x), fmaxf(v.y, fmaxf(v.z, v.w)));
        S1 += (double)fabsf(v.x);
        S1 += (double)fabsf(v.y);
        S1 += (double)fabsf(v.z);
        S1 += (double)fabsf(v.w);
    }

    // Work items of the tile: n_kpass passes over FS_KB clip ratios each, plus one light
    // pass (ternary, binary, reference energy).  Item i goes to wavefront (i + rot) % 4;
    // rot spreads the light pass over the four SIMDs from tile to tile.
    const int rot = blockIdx.x & (FS_WAVES - 1);
    const int n_items = A.n_kpass + 1;
    for (int item = (wave - rot) & (FS_WAVES - 1); item < n_items; item += FS_WAVES) {
        if (item < A.n_kpass) {
            double lo[FS_KB], rg[FS_KB], inv[FS_KB][4], dl[FS_KB][4], acc[FS_KB][4];
#pragma unroll
            for (int i = 0; i < FS_KB; ++i) {
                int k = item * FS_KB + i;
                k = k < K ? k : K - 1;
                const float p = A.grid.p[k];
                const float flo = p * mn;
                const float fhi = p * mx;
                const float frg = fhi - flo;
                lo[i] = (double)flo;
                rg[i] = (double)frg;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const float qmax = b == 0 ? 255.0f : (b == 1 ? 15.0f : (b == 2 ? 7.0f : 3.0f));
                    float d = frg / qmax;
                    const bool ok = d >= FLT_MIN;
                    d = ok ? d : 0.0f;
                    dl[i][b] = (double)d;
                    inv[i][b] = ok ? (double)(1.0f / d) : 0.0;
                    acc[i][b] = 0.0;
                }
            }
            for (int32_t c = 0; c < G; c += 4) {
                const float4 v = *reinterpret_cast<const float4*>(wrow + c);
                const double s0 = (double)s_chunk[c], s1 = (double)s_chunk[c + 1];
                const double s2 = (double)s_chunk[c + 2], s3 = (double)s_chunk[c + 3];
                score_weight((double)v.x, s0 * s0, lo, rg, inv, dl, acc);
                score_weight((double)v.y, s1 * s1, lo, rg, inv, dl, acc);
                score_weight((double)v.z, s2 * s2, lo, rg, inv, dl, acc);
                score_weight((double)v.w, s3 * s3, lo, rg, inv, dl, acc);
            }
#pragma unroll
            for (int i = 0; i < FS_KB; ++i) {
                const int k = item * FS_KB + i;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const double tot = wave_sum(valid ? acc[i][b] : 0.0);
                    if (lane == 0 && k < K) out[b * K + k] = tot;
                }
            }
        } else {
            // ternary absmean, binary sign*mean|w|, reference energy
            const float fam = (float)(S1 / (double)G);
            const bool ok = fam >= FLT_MIN;
            const double gamma = ok ? (double)fam : 0.0;
            const double ginv = ok ? (double)(1.0f / fam) : 0.0;
            const double alpha = (double)fam;
            double acc_t = 0.0, acc_b = 0.0, acc_r = 0.0;
            for (int32_t c = 0; c < G; ++c) {
                const double w = (double)wrow[c];
                const double sc = (double)s_chunk[c];
                const double a = sc * sc;
                double q = fma(w, ginv, RNE_MAGIC) - RNE_MAGIC;
                q = fmin(fmax(q, -1.0), 1.0);
                const double rt = fma(-q, gamma, w);
                acc_t = fma(a * rt, rt, acc_t);
                const double rb = fabs(w) - alpha;
                acc_b = fma(a * rb, rb, acc_b);
                acc_r = fma(a * w, w, acc_r);
            }
            const double tt = wave_sum(valid ? acc_t : 0.0);
            const double tb = wave_sum(valid ? acc_b : 0.0);
            const double tr = wave_sum(valid ? acc_r : 0.0);
            if (lane == 0) {
                out[4 * K] = tt;
                out[4 * K + 1] = tb;
                out[4 * K + 2] = tr;
            }
        }
    }
}

// Per unit: add the tiles' partial errors in tile order, pick the clip index with the
// least error for each uniform bit-width (ties to the largest index), emit fp32.
__global__ __launch_bounds__(64) void fit_score_finalize_kernel(const double* __restrict__ partial, int64_t tiles_per_unit,
                                                                 int32_t K, float* __restrict__ err,
                                                                 uint8_t* __restrict__ clip_idx,
                                                                 float* __restrict__ ref_energy) {
    __shared__ double E[4 * WINDQ_MAX_CLIP + 3];
    const int64_t u = blockIdx.x;
    const int32_t ncand = fit_score_ncand(K);
    const double* base = partial + (size_t)u * (size_t)tiles_per_unit * (size_t)ncand;
    for (int32_t cand = threadIdx.x; cand < ncand; cand += 64) {
        double acc = 0.0;
        for (int64_t t = 0; t < tiles_per_unit; ++t) acc += base[(size_t)t * ncand + cand];
        E[cand] = acc;
    }
    __syncthreads();
    const int tid = threadIdx.x;
    if (tid < 4) {
        double best = E[tid * K];
        int bk = 0;
        for (int k = 1; k < K; ++k) {
            const double e = E[tid * K + k];
            if (e <= best) {
                best = e;
                bk = k;
            }
        }
        err[u * WINDQ_N_ERR + tid] = (float)best;
        clip_idx[u * 4 + tid] = (uint8_t)bk;
    } else if (tid == 4) {
        err[u * WINDQ_N_ERR + 4] = (float)E[4 * K];
    } else if (tid == 5) {
        err[u * WINDQ_N_ERR + 5] = (float)E[4 * K + 1];
    } else if (tid == 6 && ref_energy != nullptr) {
        ref_energy[u] = (float)E[4 * K + 2];
    }
}

}  // namespace windq

using namespace windq;

extern "C" int windq_fit_score_all_bits(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows,
                                        const float* clip_grid, int32_t K, float* err, uint8_t* clip_idx,
                                        float* ref_energy, void* ws, size_t ws_bytes, void* stream) {
    FitScoreArgs A;
    int st = make_geometry(W, chunk_w, unit_rows, &A.g);
    if (st != WINDQ_OK) return st;
    if (s == nullptr || err == nullptr || clip_idx == nullptr) return WINDQ_EINVAL;
    st = check_clip_grid(clip_grid, K);
    if (st != WINDQ_OK) return st;
    if (ws == nullptr || ws_bytes < fit_score_ws_bytes(A.g, K) || !aligned(ws, 256)) return WINDQ_EWORKSPACE;
    A.W = W->data;
    A.s = s;
    A.partial = static_cast<double*>(ws);
    A.K = K;
    A.n_kpass = (K + FS_KB - 1) / FS_KB;
    for (int k = 0; k < WINDQ_MAX_CLIP; ++k) A.grid.p[k] = clip_grid[k < K ? k : K - 1];
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const size_t lds = tile_lds_bytes(chunk_w);
    const dim3 grid((unsigned)A.g.n_tiles);
    if (W->dtype == WINDQ_BF16) {
        st = ensure_lds(reinterpret_cast<const void*>(&fit_score_kernel<WINDQ_BF16>), lds);
        if (st != WINDQ_OK) return st;
        hipLaunchKernelGGL(fit_score_kernel<WINDQ_BF16>, grid, dim3(FS_THREADS), lds, hs, A);
    } else {
        st = ensure_lds(reinterpret_cast<const void*>(&fit_score_kernel<WINDQ_F32>), lds);
        if (st != WINDQ_OK) return st;
        hipLaunchKernelGGL(fit_score_kernel<WINDQ_F32>, grid, dim3(FS_THREADS), lds, hs, A);
    }
    if (hipPeekAtLastError() != hipSuccess) return WINDQ_EHIP;
    hipLaunchKernelGGL(fit_score_finalize_kernel, dim3((unsigned)A.g.U), dim3(64), 0, hs, A.partial,
                       A.g.tiles_per_unit, K, err, clip_idx, ref_energy);
    if (hipPeekAtLastError() != hipSuccess) return WINDQ_EHIP;
    return WINDQ_OK;
}
