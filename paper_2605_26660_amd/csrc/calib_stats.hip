// windq_calib_stats: per input channel activation scale from calibration activations
// (App. "Salient Weight Protection": per-channel activation scale from a calibration
// forward pass).  s_absmean[c] = mean_t |x_tc|, s_rms[c] = sqrt(mean_t x_tc^2).
//
// Pure streaming reduction over the token axis, bound by HBM.  A workgroup owns a strip
// of 512 channels and a slab of 32 tokens: each lane reads 8 consecutive channels of a
// token with 128-bit loads (64 lanes = 1 KB contiguous for bf16), the four wavefronts
// take every fourth token.  fp64 sums, combined in a fixed order: wavefronts through
// LDS, slabs by the finalize kernel.
//
// Few tokens (the calibration sets of the paper's configs: 512 per input) are a few MB, and
// two dependent launches cost more than the data: then ONE kernel does it all.  A workgroup
// owns a strip of 64 channels (8 lanes x 8) over all tokens, its 32 lane groups take every
// 32nd token, and the 32 partial sums are added in order through LDS.
#include "windq_common.hpp"
#include "windq_ws.hpp"

namespace windq {

constexpr int CALIB_THREADS = 256;
constexpr int CALIB_WAVES = CALIB_THREADS / 64;
constexpr int CALIB_COLS_PER_LANE = 8;
constexpr int CALIB_STRIP = 64 * CALIB_COLS_PER_LANE;

template <int DT>
__global__ __launch_bounds__(CALIB_THREADS) void calib_partial_kernel(const void* __restrict__ X, int64_t rows,
                                                                      int64_t cols, int64_t ld,
                                                                      double* __restrict__ partial) {
    __shared__ double red[CALIB_WAVES][2 * CALIB_COLS_PER_LANE][64];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t c0 = (int64_t)blockIdx.x * CALIB_STRIP + (int64_t)lane * CALIB_COLS_PER_LANE;
    const int64_t slab = blockIdx.y;
    const int64_t r_begin = slab * CALIB_SLAB_ROWS;
    const int64_t r_end = r_begin + CALIB_SLAB_ROWS < rows ? r_begin + CALIB_SLAB_ROWS : rows;
    double sa[CALIB_COLS_PER_LANE], sq[CALIB_COLS_PER_LANE];
#pragma unroll
    for (int j = 0; j < CALIB_COLS_PER_LANE; ++j) sa[j] = sq[j] = 0.0;
    if (c0 < cols) {
        for (int64_t r = r_begin + wave; r < r_end; r += CALIB_WAVES) {
            float v[CALIB_COLS_PER_LANE];
            const int64_t off = r * ld + c0;
            if (DT == WINDQ_BF16) {
                const uint4 raw = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(X) + off);
                v[0] = bf16_bits_to_f32(raw.x & 0xffffu); v[1] = __uint_as_float(raw.x & 0xffff0000u);
                v[2] = bf16_bits_to_f32(raw.y & 0xffffu); v[3] = __uint_as_float(raw.y & 0xffff0000u);
                v[4] = bf16_bits_to_f32(raw.z & 0xffffu); v[5] = __uint_as_float(raw.z & 0xffff0000u);
                v[6] = bf16_bits_to_f32(raw.w & 0xffffu); v[7] = __uint_as_float(raw.w & 0xffff0000u);
            } else {
                const float4* src = reinterpret_cast<const float4*>(static_cast<const float*>(X) + off);
                const float4 a = src[0], b = src[1];
                v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
                v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
            }
#pragma unroll
            for (int j = 0; j < CALIB_COLS_PER_LANE; ++j) {
                const double x = (double)v[j];
                sa[j] += fabs(x);
                sq[j] = fma(x, x, sq[j]);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < CALIB_COLS_PER_LANE; ++j) {
        red[wave][j][lane] = sa[j];
        red[wave][CALIB_COLS_PER_LANE + j][lane] = sq[j];
    }
    __syncthreads();
    if (wave == 0 && c0 < cols) {
#pragma unroll
        for (int j = 0; j < CALIB_COLS_PER_LANE; ++j) {
            double a = 0.0, q = 0.0;
#pragma unroll
            for (int w = 0; w < CALIB_WAVES; ++w) {
                a += red[w][j][lane];
                q += red[w][CALIB_COLS_PER_LANE + j][lane];
            }
            double* dst = partial + ((size_t)slab * (size_t)cols + (size_t)(c0 + j)) * 2;
            dst[0] = a;
            dst[1] = q;
        }
    }
}

constexpr int CALIB_DIRECT_LANES = 8;                                   // lanes across a strip
constexpr int CALIB_DIRECT_STRIP = CALIB_DIRECT_LANES * CALIB_COLS_PER_LANE;
constexpr int CALIB_DIRECT_GROUPS = CALIB_THREADS / CALIB_DIRECT_LANES;   // token groups
constexpr int64_t CALIB_DIRECT_MAX_ROWS = 4096;

// One activation matrix of a launch; a launch covers up to WINDQ_MAX_BATCH of them, their
// column strips numbered one matrix after the other.
struct CalibMat {
    const void* X;
    int64_t rows, cols, ld;
    float* s_absmean;
    float* s_rms;
};
struct CalibBatch {
    int32_t n;
    int64_t strip_start[WINDQ_MAX_BATCH + 1];
    CalibMat m[WINDQ_MAX_BATCH];
};

template <int DT>
__global__ __launch_bounds__(CALIB_THREADS) void calib_direct_kernel(const CalibBatch B) {
    __shared__ double red[CALIB_DIRECT_GROUPS][2][CALIB_DIRECT_STRIP + 1];
    const int mi = batch_index(B.strip_start, B.n, blockIdx.x);
    const void* __restrict__ X = B.m[mi].X;
    const int64_t rows = B.m[mi].rows, cols = B.m[mi].cols, ld = B.m[mi].ld;
    float* __restrict__ s_absmean = B.m[mi].s_absmean;
    float* __restrict__ s_rms = B.m[mi].s_rms;
    const int64_t strip = (int64_t)blockIdx.x - B.strip_start[mi];
    const int cl = threadIdx.x % CALIB_DIRECT_LANES;
    const int tg = threadIdx.x / CALIB_DIRECT_LANES;
    const int64_t c0 = strip * CALIB_DIRECT_STRIP + (int64_t)cl * CALIB_COLS_PER_LANE;
    double sa[CALIB_COLS_PER_LANE], sq[CALIB_COLS_PER_LANE];
#pragma unroll
    for (int j = 0; j < CALIB_COLS_PER_LANE; ++j) sa[j] = sq[j] = 0.0;
    if (c0 < cols) {
#pragma unroll 4
        for (int64_t r = tg; r < rows; r += CALIB_DIRECT_GROUPS) {
            float v[CALIB_COLS_PER_LANE];
            const int64_t off = r * ld + c0;
            if (DT == WINDQ_BF16) {
                const uint4 raw = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(X) + off);
                v[0] = bf16_bits_to_f32(raw.x & 0xffffu); v[1] = __uint_as_float(raw.x & 0xffff0000u);
                v[2] = bf16_bits_to_f32(raw.y & 0xffffu); v[3] = __uint_as_float(raw.y & 0xffff0000u);
                v[4] = bf16_bits_to_f32(raw.z & 0xffffu); v[5] = __uint_as_float(raw.z & 0xffff0000u);
                v[6] = bf16_bits_to_f32(raw.w & 0xffffu); v[7] = __uint_as_float(raw.w & 0xffff0000u);
            } else {
                const float4* src = reinterpret_cast<const float4*>(static_cast<const float*>(X) + off);
                const float4 a = src[0], b = src[1];
                v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
                v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
            }
#pragma unroll
            for (int j = 0; j < CALIB_COLS_PER_LANE; ++j) {
                const double x = (double)v[j];
                sa[j] += fabs(x);
                sq[j] = fma(x, x, sq[j]);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < CALIB_COLS_PER_LANE; ++j) {
        red[tg][0][cl * CALIB_COLS_PER_LANE + j] = sa[j];
        red[tg][1][cl * CALIB_COLS_PER_LANE + j] = sq[j];
    }
    __syncthreads();
    if (threadIdx.x < CALIB_DIRECT_STRIP) {
        const int64_t c = strip * CALIB_DIRECT_STRIP + threadIdx.x;
        if (c < cols) {
            double a = 0.0, q = 0.0;
#pragma unroll
            for (int g = 0; g < CALIB_DIRECT_GROUPS; ++g) {
                a += red[g][0][threadIdx.x];
                q += red[g][1][threadIdx.x];
            }
            s_absmean[c] = (float)(a / (double)rows);
            if (s_rms != nullptr) s_rms[c] = (float)sqrt(q / (double)rows);
        }
    }
}

__global__ __launch_bounds__(256) void calib_finalize_kernel(const double* __restrict__ partial, int64_t n_slabs,
                                                              int64_t rows, int64_t cols,
                                                              float* __restrict__ s_absmean,
                                                              float* __restrict__ s_rms) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= cols) return;
    double a = 0.0, q = 0.0;
    for (int64_t sl = 0; sl < n_slabs; ++sl) {
        const double* src = partial + ((size_t)sl * (size_t)cols + (size_t)c) * 2;
        a += src[0];
        q += src[1];
    }
    s_absmean[c] = (float)(a / (double)rows);
    if (s_rms != nullptr) s_rms[c] = (float)sqrt(q / (double)rows);
}

}  // namespace windq

using namespace windq;

static int calib_check(const windq_mat* X, const float* s_absmean, const void* ws, size_t ws_bytes) {
    const int st = check_matrix(X);
    if (st != WINDQ_OK) return st;
    if (s_absmean == nullptr) return WINDQ_EINVAL;
    const size_t need = calib_ws_bytes(X->rows, X->cols);
    if (ws == nullptr || ws_bytes < need || !aligned(ws, 256)) return WINDQ_EWORKSPACE;
    if (X->rows > CALIB_DIRECT_MAX_ROWS && calib_slabs(X->rows) > 65535) return WINDQ_ESHAPE;
    return WINDQ_OK;
}

// The matrices of a launch that the direct kernel takes (few tokens), all of one element type.
static int calib_direct_launch(const windq_calib_item* items, int32_t n, hipStream_t hs) {
    CalibBatch B;
    B.n = n;
    int64_t strips = 0;
    for (int32_t i = 0; i < n; ++i) {
        const windq_mat* X = items[i].X;
        B.m[i] = {X->data, X->rows, X->cols, X->ld, items[i].s_absmean, items[i].s_rms};
        B.strip_start[i] = strips;
        strips += (X->cols + CALIB_DIRECT_STRIP - 1) / CALIB_DIRECT_STRIP;
    }
    for (int32_t i = n; i <= WINDQ_MAX_BATCH; ++i) B.strip_start[i] = strips;
    for (int32_t i = n; i < WINDQ_MAX_BATCH; ++i) B.m[i] = B.m[0];
    if (strips > (int64_t)0x7fffffff) return WINDQ_ESHAPE;
    if (items[0].X->dtype == WINDQ_BF16)
        hipLaunchKernelGGL(calib_direct_kernel<WINDQ_BF16>, dim3((unsigned)strips), dim3(CALIB_THREADS), 0, hs, B);
    else
        hipLaunchKernelGGL(calib_direct_kernel<WINDQ_F32>, dim3((unsigned)strips), dim3(CALIB_THREADS), 0, hs, B);
    return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
}

static int calib_slab_launch(const windq_calib_item& it, hipStream_t hs) {
    const windq_mat* X = it.X;
    const int64_t n_slabs = calib_slabs(X->rows);
    double* partial = static_cast<double*>(it.ws);
    const dim3 grid((unsigned)((X->cols + CALIB_STRIP - 1) / CALIB_STRIP), (unsigned)n_slabs);
    if (X->dtype == WINDQ_BF16)
        hipLaunchKernelGGL(calib_partial_kernel<WINDQ_BF16>, grid, dim3(CALIB_THREADS), 0, hs, X->data, X->rows,
                           X->cols, X->ld, partial);
    else
        hipLaunchKernelGGL(calib_partial_kernel<WINDQ_F32>, grid, dim3(CALIB_THREADS), 0, hs, X->data, X->rows,
                           X->cols, X->ld, partial);
    if (hipPeekAtLastError() != hipSuccess) return WINDQ_EHIP;
    hipLaunchKernelGGL(calib_finalize_kernel, dim3((unsigned)((X->cols + 255) / 256)), dim3(256), 0, hs, partial,
                       n_slabs, X->rows, X->cols, it.s_absmean, it.s_rms);
    return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
}

extern "C" int windq_calib_stats_batch(const windq_calib_item* items, int32_t n, void* stream) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    for (int32_t i = 0; i < n; ++i) {
        if (items[i].X == nullptr) return WINDQ_EINVAL;
        const int st = calib_check(items[i].X, items[i].s_absmean, items[i].ws, items[i].ws_bytes);
        if (st != WINDQ_OK) return st;
        if (items[i].X->dtype != items[0].X->dtype) return WINDQ_EINVAL;      // one kernel per launch
    }
    hipStream_t hs = static_cast<hipStream_t>(stream);
    // matrices of few tokens share one launch; the others take their two launches each
    windq_calib_item direct[WINDQ_MAX_BATCH];
    int32_t nd = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (items[i].X->rows <= CALIB_DIRECT_MAX_ROWS) {
            direct[nd++] = items[i];
        } else {
            const int st = calib_slab_launch(items[i], hs);
            if (st != WINDQ_OK) return st;
        }
    }
    return nd > 0 ? calib_direct_launch(direct, nd, hs) : WINDQ_OK;
}

extern "C" int windq_calib_stats(const windq_mat* X, float* s_absmean, float* s_rms, void* ws, size_t ws_bytes,
                                 void* stream) {
    const windq_calib_item it = {X, s_absmean, s_rms, ws, ws_bytes};
    if (X == nullptr) return WINDQ_EINVAL;
    return windq_calib_stats_batch(&it, 1, stream);
}
