// windq_dequant_plan: the way back from the packed artefact.  Unpacks the codes of a plan,
// reconstructs every weight from the stored per-group scale and offset, and recomputes the
// activation-weighted reconstruction error per unit from the artefact alone: the same number
// windq_fit_score_all_bits reported for the plan's bit-width and clip index (Sec. 3.5 scores a
// fit by its reconstruction error; this closes the loop codes -> error), and the first piece of
// a path that serves the quantized weights.
//   uniform:  w_hat = offset + code * scale     ternary: scale * (trit - 1)     binary: +-scale
// Errors use w_hat in fp64 from the stored fp32 numbers, as the fit does; the optional fp32
// output is one fused multiply-add.  One wavefront per 64-row tile, one lane per row: a row's
// packed bytes are contiguous, so a lane walks its own byte stream.  Reads 2 bytes per weight
// plus the codes; bound by HBM.
#include "windq_common.hpp"
#include "windq_ws.hpp"

namespace windq {

struct DequantArgs {
    const void* W;
    const float* s;
    const uint8_t* mask;       // or null
    int64_t mask_ld;
    const uint8_t* action;
    const int64_t* code_off;
    const uint8_t* codes;
    int64_t codes_bytes;
    const float* scale;
    const float* offset;
    Geometry g;
    float* what;               // [rows][what_ld] or null
    int64_t what_ld;
    double* part;              // [n_tiles]
};

__device__ __forceinline__ int64_t dq_bytes_per_group(int a, int G) {
    switch (a) {
        case 1: return G;
        case 2: return G >> 1;
        case 3: return (G * 3) >> 3;
        case 4: return G >> 2;
        case 5: return (G + 4) / 5;
        case 6: return G >> 3;
        default: return 0;
    }
}

template <int DT>
__global__ __launch_bounds__(64) void dequant_tile_kernel(const DequantArgs A) {
    extern __shared__ char smem[];
    const TileCoord tc = tile_coord(A.g, blockIdx.x);
    const int32_t G = A.g.chunk_w;
    constexpr int EB = Elem<DT>::bytes;
    const int32_t row_bytes = G * EB + 16;
    float* scol = reinterpret_cast<float*>(smem + TILE_ROWS * row_bytes);
    const int lane = threadIdx.x;
    load_tile_raw<DT>(A.W, A.g.ld, tc, G, smem);
    for (int32_t c = lane; c < G; c += 64) scol[c] = A.s[tc.col0 + c];
    __syncthreads();

    int a = A.action[tc.u];
    if (a >= WINDQ_N_ACTIONS) a = 0;
    const int64_t bpg = dq_bytes_per_group(a, G);
    const int64_t base = A.code_off[tc.u];
    if (base < 0 || base + bpg * A.g.R_u > A.codes_bytes) a = 0;      // an entry that points outside the stream reads nothing

    double acc = 0.0;
    if (lane < tc.nrows) {
        const char* wrow = smem + lane * row_bytes;
        const int64_t row = tc.row0 + lane;
        const int64_t gidx = tc.u * A.g.R_u + tc.lrow0 + lane;
        const float sc = a != 0 ? A.scale[gidx] : 0.0f;
        const float of = a != 0 ? A.offset[gidx] : 0.0f;
        const uint8_t* __restrict__ src = A.codes + base + (tc.lrow0 + lane) * bpg;
        const uint8_t* __restrict__ mrow = A.mask != nullptr ? A.mask + row * A.mask_ld + (tc.col0 >> 3) : nullptr;
        float* __restrict__ orow = A.what != nullptr ? A.what + row * A.what_ld + tc.col0 : nullptr;
        const int bits = a == 1 ? 8 : (a == 2 ? 4 : (a == 3 ? 3 : (a == 4 ? 2 : 1)));
        for (int32_t c = 0; c < G; c += 8) {
            float w[8];
            read8<DT>(wrow, c, w);
            const uint32_t m = mrow != nullptr ? mrow[c >> 3] : 0u;
            uint32_t stored[8];
            if (a == 5) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int32_t i = c + j;
                    const uint32_t byte = src[i / 5];
                    const int pos = i % 5;
                    const uint32_t div = pos == 0 ? 1u : (pos == 1 ? 3u : (pos == 2 ? 9u : (pos == 3 ? 27u : 81u)));
                    stored[j] = (byte / div) % 3u;
                }
            } else if (a != 0) {
                uint64_t v = 0;
                const uint8_t* p = src + (c >> 3) * bits;          // eight codes = `bits` bytes
                for (int b = 0; b < bits; ++b) v |= (uint64_t)p[b] << (8 * b);
#pragma unroll
                for (int j = 0; j < 8; ++j) stored[j] = (uint32_t)(v >> (j * bits)) & ((1u << bits) - 1u);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool prot = ((m >> j) & 1u) != 0u;
                float wh = w[j];                                      // a skip unit keeps its weights
                if (a != 0) {
                    double whd;
                    if (a <= 4) {
                        wh = fmaf((float)stored[j], sc, of);
                        whd = (double)of + (double)stored[j] * (double)sc;
                    } else if (a == 5) {
                        wh = sc * ((float)stored[j] - 1.0f);
                        whd = (double)wh;
                    } else {
                        wh = stored[j] != 0u ? sc : -sc;
                        whd = (double)wh;
                    }
                    if (prot) {
                        wh = 0.0f;                                    // lives in the INT8 side stream
                    } else {
                        const double d = (double)w[j] - whd;
                        const double ac = (double)scol[c + j] * (double)scol[c + j];
                        acc = fma(ac * d, d, acc);
                    }
                }
                if (orow != nullptr) orow[c + j] = wh;
            }
        }
    }
    acc = wave_sum(acc);
    if (lane == 0) A.part[(size_t)tc.u * (size_t)A.g.tiles_per_unit + (size_t)tc.t] = acc;
}

__global__ __launch_bounds__(64) void dequant_finalize_kernel(const double* __restrict__ part, const Geometry g,
                                                             float* __restrict__ err) {
    const int64_t u = (int64_t)blockIdx.x * 64 + threadIdx.x;
    if (u >= g.U) return;
    double t = 0.0;
    for (int64_t i = 0; i < g.tiles_per_unit; ++i) t += part[(size_t)u * (size_t)g.tiles_per_unit + (size_t)i];
    err[u] = (float)t;
}

}  // namespace windq

using namespace windq;

extern "C" int windq_dequant_plan(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows,
                                  const uint8_t* mask, const uint8_t* action, const int64_t* code_off,
                                  const uint8_t* codes, size_t codes_bytes, const float* scale, const float* offset,
                                  float* err, float* w_hat, void* ws, size_t ws_bytes, void* stream) {
    DequantArgs A;
    int st = make_geometry(W, chunk_w, unit_rows, &A.g);
    if (st != WINDQ_OK) return st;
    if (s == nullptr || action == nullptr || code_off == nullptr || scale == nullptr || offset == nullptr)
        return WINDQ_EINVAL;
    if (codes == nullptr && codes_bytes != 0) return WINDQ_EINVAL;
    if (err == nullptr && w_hat == nullptr) return WINDQ_EINVAL;
    if (!aligned(code_off, 8) || (w_hat != nullptr && !aligned(w_hat, 4))) return WINDQ_EINVAL;
    if (ws == nullptr || ws_bytes < unit_saliency_ws_bytes(A.g) || !aligned(ws, 256)) return WINDQ_EWORKSPACE;
    A.W = W->data;
    A.s = s;
    A.mask = mask;
    A.mask_ld = W->cols / 8;
    A.action = action;
    A.code_off = code_off;
    A.codes = codes;
    A.codes_bytes = (int64_t)codes_bytes;
    A.scale = scale;
    A.offset = offset;
    A.what = w_hat;
    A.what_ld = W->cols;
    A.part = static_cast<double*>(ws);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const size_t lds = raw_tile_lds_bytes(W->dtype, chunk_w) + (size_t)chunk_w * sizeof(float);
    const dim3 tiles((unsigned)A.g.n_tiles);
    if (W->dtype == WINDQ_BF16) {
        st = ensure_lds(reinterpret_cast<const void*>(&dequant_tile_kernel<WINDQ_BF16>), lds);
        if (st != WINDQ_OK) return st;
        hipLaunchKernelGGL(dequant_tile_kernel<WINDQ_BF16>, tiles, dim3(64), lds, hs, A);
    } else {
        st = ensure_lds(reinterpret_cast<const void*>(&dequant_tile_kernel<WINDQ_F32>), lds);
        if (st != WINDQ_OK) return st;
        hipLaunchKernelGGL(dequant_tile_kernel<WINDQ_F32>, tiles, dim3(64), lds, hs, A);
    }
    if (err != nullptr)
        hipLaunchKernelGGL(dequant_finalize_kernel, dim3((unsigned)((A.g.U + 63) / 64)), dim3(64), 0, hs, A.part, A.g, err);
    return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
}
