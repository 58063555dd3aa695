// windq_unit_features: the tensor-statistics part of the controller's state (Table 1):
// dims 0-4 (mean, std, mean|w|, fraction |w| < 1e-6, fraction |w| > 0.5 P99) for every
// unit, and dims 9-11 (mean, std, max of the activation scale over the unit's chunk).
//
// Everything but P99 is a streaming reduction (fp64 sums, integer counts).  P99 is the
// exact nearest-rank order statistic of |w|, found by most-significant-digit radix
// selection on the bit pattern of |w| (monotone in |w| for non-negative floats):
// bf16 keys have 15 bits -> digits of 11 + 4 bits; fp32 keys 31 bits -> 11 + 11 + 9.
// The first digit (exponent + 3 mantissa bits) spreads Gaussian-like weights over
// enough bins to keep LDS atomics from piling up on one address.  Each digit costs one
// pass over W; the first shares its pass with the moments, later passes touch the
// histogram only for the few keys that match the prefix, and a last pass counts
// |w| > 0.5 P99 (as 2|w| > P99, exact in fp32).  All passes after the first re-read a
// matrix that was just streamed, so for matrices up to the 256 MB last-level cache they
// are served on chip.  Integer atomics only: results are bit-reproducible.
#include <math.h>

#include "windq_common.hpp"
#include "windq_ws.hpp"

namespace windq {

constexpr int FT_THREADS = 256;

struct DigitPlan {
    int32_t n_levels;
    int32_t shift[3];
    int32_t bits[3];
};

struct FeatArgs {
    const void* W;
    const float* s;
    float* feat;
    double* moments;
    uint32_t* above;
    uint32_t* hist;
    FeatSel* sel;
    Geometry g;
    DigitPlan dp;
    float sparse_thr;   // smallest fp32 that is >= 1e-6: (|w| < 1e-6) == (|w| < sparse_thr) for fp32 |w|
    uint64_t rank;      // ceil(0.99 n), 1-based
};

// Loads 8 consecutive elements as the bit pattern of |w| widened to fp32 layout and the
// signed fp32 value.
template <int DT>
__device__ __forceinline__ void load8(const void* __restrict__ data, int64_t off, float (&w)[8]) {
    if (DT == WINDQ_BF16) {
        const uint4 raw = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(data) + off);
        w[0] = bf16_bits_to_f32(raw.x & 0xffffu); w[1] = __uint_as_float(raw.x & 0xffff0000u);
        w[2] = bf16_bits_to_f32(raw.y & 0xffffu); w[3] = __uint_as_float(raw.y & 0xffff0000u);
        w[4] = bf16_bits_to_f32(raw.z & 0xffffu); w[5] = __uint_as_float(raw.z & 0xffff0000u);
        w[6] = bf16_bits_to_f32(raw.w & 0xffffu); w[7] = __uint_as_float(raw.w & 0xffff0000u);
    } else {
        const float4* src = reinterpret_cast<const float4*>(static_cast<const float*>(data) + off);
        const float4 a = src[0], b = src[1];
        w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w;
        w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
    }
}

// Selection key of a weight: the magnitude bits, 15 for bf16 (fp32 pattern >> 16), 31 for fp32.
template <int DT>
__device__ __forceinline__ uint32_t key_of(float w) {
    const uint32_t b = __float_as_uint(w) & 0x7fffffffu;
    return DT == WINDQ_BF16 ? (b >> 16) : b;
}
template <int DT>
__device__ __forceinline__ float value_of_key(uint32_t key) {
    return __uint_as_float(DT == WINDQ_BF16 ? (key << 16) : key);
}

__global__ __launch_bounds__(256) void feat_init_kernel(uint32_t* __restrict__ hist, FeatSel* __restrict__ sel,
                                                         int64_t U, uint64_t rank) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < U * FEAT_BINS) hist[i] = 0;
    if (i < U) {
        sel[i].prefix = 0;
        sel[i].pad = 0;
        sel[i].rank = rank;
    }
}

// Pass over one tile.  LEVEL 0: moments + histogram of the first digit.  LEVEL > 0:
// histogram of digit `level` among keys whose higher digits equal the unit's prefix.
// LEVEL < 0: count of 2|w| > P99.
template <int DT, int MODE>   // MODE 0: first pass, 1: later digit, 2: count above half P99
__global__ __launch_bounds__(FT_THREADS) void feat_pass_kernel(const FeatArgs A, const int32_t level) {
    __shared__ uint32_t lhist[FEAT_BINS];
    __shared__ double red[FT_THREADS / 64][4];
    const TileCoord tc = tile_coord(A.g, blockIdx.x);
    const int32_t G = A.g.chunk_w;
    const int32_t pieces = G >> 3;
    const int32_t total = tc.nrows * pieces;
    const int32_t shift = MODE == 2 ? 0 : A.dp.shift[level];
    const int32_t nbins = MODE == 2 ? 0 : (1 << A.dp.bits[level]);
    const uint32_t mask = (uint32_t)nbins - 1u;
    if (MODE != 2) {
        for (int32_t b = threadIdx.x; b < nbins; b += FT_THREADS) lhist[b] = 0;
        __syncthreads();
    }
    uint32_t prefix = 0;
    float p99 = 0.0f;
    if (MODE == 1) prefix = A.sel[tc.u].prefix;
    if (MODE == 2) p99 = value_of_key<DT>(A.sel[tc.u].prefix);

    double sw = 0.0, sw2 = 0.0, sabs = 0.0;
    uint32_t cnt = 0;
    for (int32_t i = threadIdx.x; i < total; i += FT_THREADS) {
        const int32_t r = i / pieces;
        const int32_t pc = i - r * pieces;
        float w[8];
        load8<DT>(A.W, (tc.row0 + r) * A.g.ld + tc.col0 + (int64_t)pc * 8, w);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float aw = fabsf(w[j]);
            if (MODE == 0) {
                const double x = (double)w[j];
                sw += x;
                sw2 = fma(x, x, sw2);
                sabs += (double)aw;
                cnt += aw < A.sparse_thr ? 1u : 0u;
                atomicAdd(&lhist[key_of<DT>(w[j]) >> shift], 1u);
            } else if (MODE == 1) {
                const uint32_t key = key_of<DT>(w[j]);
                if ((key >> (shift + A.dp.bits[level])) == prefix) atomicAdd(&lhist[(key >> shift) & mask], 1u);
            } else {
                cnt += 2.0f * aw > p99 ? 1u : 0u;
            }
        }
    }

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t tile_slot = (size_t)tc.u * (size_t)A.g.tiles_per_unit + (size_t)tc.t;
    if (MODE == 0) {
        const double r0 = wave_sum(sw), r1 = wave_sum(sw2), r2 = wave_sum(sabs);
        const double r3 = (double)wave_sum_u64((unsigned long long)cnt);
        if (lane == 0) {
            red[wave][0] = r0; red[wave][1] = r1; red[wave][2] = r2; red[wave][3] = r3;
        }
        __syncthreads();
        if (threadIdx.x < 4) {
            double acc = 0.0;
            for (int w = 0; w < FT_THREADS / 64; ++w) acc += red[w][threadIdx.x];
            A.moments[tile_slot * 4 + threadIdx.x] = acc;
        }
    } else if (MODE == 2) {
        const double r3 = (double)wave_sum_u64((unsigned long long)cnt);
        if (lane == 0) red[wave][0] = r3;
        __syncthreads();
        if (threadIdx.x == 0) {
            double acc = 0.0;
            for (int w = 0; w < FT_THREADS / 64; ++w) acc += red[w][0];
            A.above[tile_slot] = (uint32_t)acc;
        }
    }
    if (MODE != 2) {
        __syncthreads();
        uint32_t* __restrict__ gh = A.hist + (size_t)tc.u * FEAT_BINS;
        for (int32_t b = threadIdx.x; b < nbins; b += FT_THREADS) {
            const uint32_t v = lhist[b];
            if (v != 0) atomicAdd(&gh[b], v);
        }
    }
}

// Per unit: find the bin of the current digit that holds the wanted rank, extend the
// prefix, reduce the rank to a rank inside that bin, and clear the histogram for the
// next digit.
__global__ __launch_bounds__(256) void feat_select_kernel(uint32_t* __restrict__ hist, FeatSel* __restrict__ sel,
                                                           const int32_t bits) {
    __shared__ uint64_t part[256];
    __shared__ uint32_t chosen_chunk;
    __shared__ uint64_t chosen_before;
    const int64_t u = blockIdx.x;
    const int32_t nbins = 1 << bits;
    const int32_t per = (nbins + 255) / 256;
    uint32_t* __restrict__ h = hist + (size_t)u * FEAT_BINS;
    const int32_t b0 = threadIdx.x * per;
    uint64_t local = 0;
    for (int32_t b = b0; b < b0 + per && b < nbins; ++b) local += h[b];
    part[threadIdx.x] = local;
    __syncthreads();
    const uint64_t rank = sel[u].rank;
    if (threadIdx.x == 0) {
        uint64_t cum = 0;
        uint32_t ci = 255;
        for (uint32_t i = 0; i < 256; ++i) {
            if (cum + part[i] >= rank) {
                ci = i;
                break;
            }
            cum += part[i];
        }
        chosen_chunk = ci;
        chosen_before = cum;
    }
    __syncthreads();
    if (threadIdx.x == chosen_chunk) {
        uint64_t cum = chosen_before;
        int32_t bin = b0;
        for (int32_t b = b0; b < b0 + per && b < nbins; ++b) {
            bin = b;
            if (cum + h[b] >= rank) break;
            cum += h[b];
        }
        sel[u].prefix = (sel[u].prefix << bits) | (uint32_t)bin;
        sel[u].rank = rank - cum;
    }
    __syncthreads();
    for (int32_t b = b0; b < b0 + per && b < nbins; ++b) h[b] = 0;
}

// Per unit: combine the tiles' partial sums in tile order and emit the eight features.
__global__ __launch_bounds__(64) void feat_finalize_kernel(const FeatArgs A) {
    const int64_t u = blockIdx.x;
    const int lane = threadIdx.x;
    const int64_t T = A.g.tiles_per_unit;
    double m[4] = {0.0, 0.0, 0.0, 0.0};
    double ab = 0.0;
    for (int64_t t = lane; t < T; t += 64) {
        const double* src = A.moments + ((size_t)u * (size_t)T + (size_t)t) * 4;
        m[0] += src[0]; m[1] += src[1]; m[2] += src[2]; m[3] += src[3];
        ab += (double)A.above[(size_t)u * (size_t)T + (size_t)t];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) m[j] = wave_sum(m[j]);
    ab = wave_sum(ab);
    const int32_t G = A.g.chunk_w;
    const float* __restrict__ sc = A.s + (u % A.g.n_chunks) * G;
    double ssum = 0.0;
    float smax = sc[0];
    for (int32_t c = lane; c < G; c += 64) {
        ssum += (double)sc[c];
        smax = fmaxf(smax, sc[c]);
    }
    ssum = wave_sum(ssum);
#pragma unroll
    for (int mm = 32; mm >= 1; mm >>= 1) smax = fmaxf(smax, __shfl_xor(smax, mm, 64));
    const double smean = ssum / (double)G;
    double sdev = 0.0;
    for (int32_t c = lane; c < G; c += 64) {
        const double d = (double)sc[c] - smean;
        sdev = fma(d, d, sdev);
    }
    sdev = wave_sum(sdev);
    if (lane == 0) {
        const double n = (double)A.g.R_u * (double)G;
        const double mean = m[0] / n;
        double var = m[1] / n - mean * mean;
        var = var > 0.0 ? var : 0.0;
        float* f = A.feat + u * WINDQ_N_FEAT;
        f[0] = (float)mean;
        f[1] = (float)sqrt(var);
        f[2] = (float)(m[2] / n);
        f[3] = (float)(m[3] / n);
        f[4] = (float)(ab / n);
        f[5] = (float)smean;
        f[6] = (float)sqrt(sdev / (double)G);
        f[7] = smax;
    }
}

template <int DT>
static int launch_features(const FeatArgs& A, hipStream_t hs) {
    const dim3 tiles((unsigned)A.g.n_tiles), units((unsigned)A.g.U);
    const int64_t n_init = A.g.U * FEAT_BINS;
    hipLaunchKernelGGL(feat_init_kernel, dim3((unsigned)((n_init + 255) / 256)), dim3(256), 0, hs, A.hist, A.sel,
                       A.g.U, A.rank);
    hipLaunchKernelGGL((feat_pass_kernel<DT, 0>), tiles, dim3(FT_THREADS), 0, hs, A, 0);
    hipLaunchKernelGGL(feat_select_kernel, units, dim3(256), 0, hs, A.hist, A.sel, A.dp.bits[0]);
    for (int32_t l = 1; l < A.dp.n_levels; ++l) {
        hipLaunchKernelGGL((feat_pass_kernel<DT, 1>), tiles, dim3(FT_THREADS), 0, hs, A, l);
        hipLaunchKernelGGL(feat_select_kernel, units, dim3(256), 0, hs, A.hist, A.sel, A.dp.bits[l]);
    }
    hipLaunchKernelGGL((feat_pass_kernel<DT, 2>), tiles, dim3(FT_THREADS), 0, hs, A, 0);
    hipLaunchKernelGGL(feat_finalize_kernel, units, dim3(64), 0, hs, A);
    return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
}

}  // namespace windq

using namespace windq;

extern "C" int windq_unit_features(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows, float* feat,
                                   void* ws, size_t ws_bytes, void* stream) {
    FeatArgs A;
    const int st = make_geometry(W, chunk_w, unit_rows, &A.g);
    if (st != WINDQ_OK) return st;
    if (s == nullptr || feat == nullptr) return WINDQ_EINVAL;
    const FeatLayout L = features_layout(A.g);
    if (ws == nullptr || ws_bytes < L.total || !aligned(ws, 256)) return WINDQ_EWORKSPACE;
    if ((uint64_t)A.g.R_u * (uint64_t)chunk_w > (uint64_t)0xffffffffu) return WINDQ_ESHAPE;   // u32 bin counts
    char* base = static_cast<char*>(ws);
    A.W = W->data;
    A.s = s;
    A.feat = feat;
    A.moments = reinterpret_cast<double*>(base + L.moments);
    A.above = reinterpret_cast<uint32_t*>(base + L.above);
    A.hist = reinterpret_cast<uint32_t*>(base + L.hist);
    A.sel = reinterpret_cast<FeatSel*>(base + L.sel);
    if (W->dtype == WINDQ_BF16) {
        A.dp.n_levels = 2;
        A.dp.shift[0] = 4;  A.dp.bits[0] = 11;
        A.dp.shift[1] = 0;  A.dp.bits[1] = 4;
        A.dp.shift[2] = 0;  A.dp.bits[2] = 0;
    } else {
        A.dp.n_levels = 3;
        A.dp.shift[0] = 20; A.dp.bits[0] = 11;
        A.dp.shift[1] = 9;  A.dp.bits[1] = 11;
        A.dp.shift[2] = 0;  A.dp.bits[2] = 9;
    }
    float thr = (float)1e-6;
    if ((double)thr < 1e-6) thr = nextafterf(thr, INFINITY);
    A.sparse_thr = thr;
    const uint64_t n = (uint64_t)A.g.R_u * (uint64_t)chunk_w;
    A.rank = (99 * n + 99) / 100;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    return W->dtype == WINDQ_BF16 ? launch_features<WINDQ_BF16>(A, hs) : launch_features<WINDQ_F32>(A, hs);
}
