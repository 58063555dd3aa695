// windq_apply_plan: materialise a mixed-precision plan as packed codes plus per-group
// scale and offset (Sec. 3.3: the environment applies the selected quantization to the
// unit; Sec. 3.5: the engine applies the operator of the chosen bit-width).
//
// Codes and stored scales are DEFINED by a short sequence of correctly rounded fp32
// operations (see windq.h); this file is compiled with floating-point contraction off so
// that each written operation is exactly one IEEE operation.  The sum of |w| of a group
// is accumulated in fp64 in column order (exact for bf16 inputs).
//
// Streaming kernel, bound by HBM: reads 2 (bf16) or 4 (fp32) bytes per weight once,
// writes b/8 bytes of codes per weight and 8 bytes per group.  One wavefront per tile of
// 64 rows x one chunk.  The tile is loaded with coalesced 128-bit loads into LDS in the
// input's own element type (17 KB for bf16 at chunk 128: nine workgroups per CU, whose
// loads overlap each other's arithmetic).  Each lane quantizes and packs its own row, so
// ternary base-3 bytes and 3-bit streams need no cross-lane regrouping, and writes the
// packed bytes back INTO ITS OWN ROW of the tile: packed output never overtakes the read
// position (b/8 <= element bytes).  Rows of a unit are consecutive in the code stream, so
// the 64 packed rows are then copied to one contiguous byte range with coalesced stores.
#include <float.h>

#include "windq_common.hpp"
#include "windq_ws.hpp"

namespace windq {

constexpr int AP_THREADS = 64;

struct ApplyArgs {
    const void* W;
    const uint8_t* action;
    const uint8_t* clip_idx;   // may be null
    const int64_t* code_off;
    uint8_t* codes;
    int64_t codes_bytes;
    float* scale;
    float* offset;
    Geometry g;
    int32_t K;
    ClipGrid grid;
};

__device__ __forceinline__ int64_t dev_bytes_per_group(int a, int G) {
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

// Eight BITS-bit codes -> BITS bytes, LSB first, stored at dst (which is aligned to the
// natural width of the store used).
template <int BITS>
__device__ __forceinline__ void store_codes8(uint8_t* dst, const uint32_t (&c)[8]) {
    uint64_t v = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) v |= (uint64_t)c[j] << (j * BITS);
    if (BITS == 8) {
        *reinterpret_cast<uint2*>(dst) = make_uint2((uint32_t)v, (uint32_t)(v >> 32));
    } else if (BITS == 4) {
        *reinterpret_cast<uint32_t*>(dst) = (uint32_t)v;
    } else if (BITS == 2) {
        *reinterpret_cast<uint16_t*>(dst) = (uint16_t)v;
    } else if (BITS == 3) {
        dst[0] = (uint8_t)v;
        dst[1] = (uint8_t)(v >> 8);
        dst[2] = (uint8_t)(v >> 16);
    } else {
        dst[0] = (uint8_t)v;
    }
}

// Uniform BITS-bit quantizer of one group, normative fp32 steps.
template <int DT, int BITS>
__device__ __forceinline__ void quantize_uniform(const char* wrow, int32_t G, float p, uint8_t* dst, float* scale_out,
                                                 float* offset_out) {
    float w[8];
    read8<DT>(wrow, 0, w);
    float mn = w[0], mx = w[0];
    for (int32_t c = 0; c < G; c += 8) {
        read8<DT>(wrow, c, w);
        mn = fminf(fminf(fminf(mn, w[0]), fminf(w[1], w[2])), fminf(fminf(w[3], w[4]), fminf(w[5], fminf(w[6], w[7]))));
        mx = fmaxf(fmaxf(fmaxf(mx, w[0]), fmaxf(w[1], w[2])), fmaxf(fmaxf(w[3], w[4]), fmaxf(w[5], fmaxf(w[6], w[7]))));
    }
    const float qmax = (float)((1 << BITS) - 1);
    const float lo = p * mn;
    const float hi = p * mx;
    const float rg = hi - lo;
    float d = rg / qmax;
    const bool ok = d >= FLT_MIN;
    d = ok ? d : 0.0f;
    const float inv = ok ? 1.0f / d : 0.0f;
    *scale_out = d;
    *offset_out = lo;
    for (int32_t c = 0; c < G; c += 8) {
        read8<DT>(wrow, c, w);
        uint32_t code[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float u = w[j] - lo;
            const float t = u * inv;
            const float q = __builtin_amdgcn_fmed3f(__builtin_rintf(t), 0.0f, qmax);
            code[j] = (uint32_t)q;
        }
        store_codes8<BITS>(dst + (c >> 3) * BITS, code);
    }
}

// Sum of |w| of a group in fp64 in column order (exact for bf16 inputs).
template <int DT>
__device__ __forceinline__ double group_abs_sum(const char* wrow, int32_t G) {
    double S1 = 0.0;
    for (int32_t c = 0; c < G; c += 8) {
        float w[8];
        read8<DT>(wrow, c, w);
#pragma unroll
        for (int j = 0; j < 8; ++j) S1 += (double)fabsf(w[j]);
    }
    return S1;
}

template <int DT>
__device__ __forceinline__ void quantize_ternary(const char* wrow, int32_t G, uint8_t* dst, float* scale_out) {
    float gamma = (float)(group_abs_sum<DT>(wrow, G) / (double)G);
    const bool ok = gamma >= FLT_MIN;
    gamma = ok ? gamma : 0.0f;
    const float inv = ok ? 1.0f / gamma : 0.0f;
    *scale_out = gamma;
    uint32_t byte = 0, mul = 1;
    int32_t nb = 0;
    for (int32_t c = 0; c < G; c += 8) {
        float w[8];
        read8<DT>(wrow, c, w);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float t = w[j] * inv;
            const float q = __builtin_amdgcn_fmed3f(__builtin_rintf(t), -1.0f, 1.0f);
            byte += (uint32_t)((int32_t)q + 1) * mul;
            mul *= 3;
            if (mul == 243) {
                dst[nb++] = (uint8_t)byte;
                byte = 0;
                mul = 1;
            }
        }
    }
    if (mul != 1) dst[nb] = (uint8_t)byte;
}

template <int DT>
__device__ __forceinline__ void quantize_binary(const char* wrow, int32_t G, uint8_t* dst, float* scale_out) {
    *scale_out = (float)(group_abs_sum<DT>(wrow, G) / (double)G);
    for (int32_t c = 0; c < G; c += 8) {
        float w[8];
        read8<DT>(wrow, c, w);
        uint32_t byte = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) byte |= (w[j] >= 0.0f ? 1u : 0u) << j;
        dst[c >> 3] = (uint8_t)byte;
    }
}

template <int DT>
__global__ __launch_bounds__(AP_THREADS) void apply_plan_kernel(const ApplyArgs A) {
    extern __shared__ char tile[];
    const TileCoord tc = tile_coord(A.g, blockIdx.x);
    const int32_t G = A.g.chunk_w;
    const int lane = threadIdx.x;
    const bool valid = lane < tc.nrows;
    const int64_t gidx = tc.u * A.g.R_u + tc.lrow0 + lane;

    // Plan entry of the unit (uniform over the workgroup), with the guards that turn a
    // malformed entry into "skip" instead of a stray write.
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
        return;
    }

    load_tile_raw<DT>(A.W, A.g.ld, tc, G, tile);
    __syncthreads();

    const int32_t row_bytes = G * Elem<DT>::bytes + 16;
    char* wrow = tile + lane * row_bytes;
    if (valid) {
        float p = 1.0f;
        if (a <= 4 && A.clip_idx != nullptr) {
            int k = A.clip_idx[tc.u * 4 + (a - 1)];
            k = k < A.K ? k : A.K - 1;
            p = A.grid.p[k];
        }
        uint8_t* dst = reinterpret_cast<uint8_t*>(wrow);   // packed in place, behind the read position
        float sc = 0.0f, of = 0.0f;
        switch (a) {
            case 1: quantize_uniform<DT, 8>(wrow, G, p, dst, &sc, &of); break;
            case 2: quantize_uniform<DT, 4>(wrow, G, p, dst, &sc, &of); break;
            case 3: quantize_uniform<DT, 3>(wrow, G, p, dst, &sc, &of); break;
            case 4: quantize_uniform<DT, 2>(wrow, G, p, dst, &sc, &of); break;
            case 5: quantize_ternary<DT>(wrow, G, dst, &sc); break;
            default: quantize_binary<DT>(wrow, G, dst, &sc); break;
        }
        A.scale[gidx] = sc;
        A.offset[gidx] = of;
    }
    __syncthreads();

    // Copy the tile's packed rows (bpg bytes each, row_bytes apart in LDS) to the contiguous
    // range of the code stream, in elements of the widest size that divides bpg.
    const int32_t e = (bpg & 15) == 0 ? 16 : ((bpg & 3) == 0 ? 4 : ((bpg & 1) == 0 ? 2 : 1));
    const int32_t total = tc.nrows * (int32_t)bpg;
    uint8_t* __restrict__ out = A.codes + base + tc.lrow0 * bpg;
    int32_t byte = lane * e;
    int32_t row = byte / (int32_t)bpg;
    int32_t col = byte - row * (int32_t)bpg;
    for (; byte < total; byte += AP_THREADS * e) {
        const char* src = tile + row * row_bytes + col;
        if (e == 16) *reinterpret_cast<uint4*>(out + byte) = *reinterpret_cast<const uint4*>(src);
        else if (e == 4) *reinterpret_cast<uint32_t*>(out + byte) = *reinterpret_cast<const uint32_t*>(src);
        else if (e == 2) *reinterpret_cast<uint16_t*>(out + byte) = *reinterpret_cast<const uint16_t*>(src);
        else out[byte] = *reinterpret_cast<const uint8_t*>(src);
        col += AP_THREADS * e;
        while (col >= (int32_t)bpg) {
            col -= (int32_t)bpg;
            ++row;
        }
    }
    // zero the padding that rounds the unit's payload up to 16 bytes
    if (padded != payload && tc.t == A.g.tiles_per_unit - 1 && lane < padded - payload)
        A.codes[base + payload + lane] = 0;
}

}  // namespace windq

using namespace windq;

extern "C" int windq_apply_plan(const windq_mat* W, int32_t chunk_w, int64_t unit_rows, const uint8_t* action,
                                const uint8_t* clip_idx, const float* clip_grid, int32_t K, const int64_t* code_off,
                                uint8_t* codes, size_t codes_bytes, float* scale, float* offset, void* ws,
                                size_t ws_bytes, void* stream) {
    ApplyArgs A;
    int st = make_geometry(W, chunk_w, unit_rows, &A.g);
    if (st != WINDQ_OK) return st;
    if (action == nullptr || code_off == nullptr || scale == nullptr || offset == nullptr) return WINDQ_EINVAL;
    if (codes == nullptr && codes_bytes != 0) return WINDQ_EINVAL;
    if (codes != nullptr && !aligned(codes, 16)) return WINDQ_EINVAL;
    if (!aligned(code_off, 8)) return WINDQ_EINVAL;
    if (clip_idx != nullptr || clip_grid != nullptr) {
        st = check_clip_grid(clip_grid, K);
        if (st != WINDQ_OK) return st;
    } else {
        K = 1;
    }
    if (ws == nullptr || ws_bytes < apply_ws_bytes(A.g) || !aligned(ws, 256)) return WINDQ_EWORKSPACE;
    A.W = W->data;
    A.action = action;
    A.clip_idx = clip_grid != nullptr ? clip_idx : nullptr;
    A.code_off = code_off;
    A.codes = codes;
    A.codes_bytes = (int64_t)codes_bytes;
    A.scale = scale;
    A.offset = offset;
    A.K = K;
    for (int k = 0; k < WINDQ_MAX_CLIP; ++k) A.grid.p[k] = clip_grid != nullptr ? clip_grid[k < K ? k : K - 1] : 1.0f;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const size_t lds = raw_tile_lds_bytes(W->dtype, chunk_w);
    const dim3 grid((unsigned)A.g.n_tiles);
    if (W->dtype == WINDQ_BF16) {
        st = ensure_lds(reinterpret_cast<const void*>(&apply_plan_kernel<WINDQ_BF16>), lds);
        if (st != WINDQ_OK) return st;
        hipLaunchKernelGGL(apply_plan_kernel<WINDQ_BF16>, grid, dim3(AP_THREADS), lds, hs, A);
    } else {
        st = ensure_lds(reinterpret_cast<const void*>(&apply_plan_kernel<WINDQ_F32>), lds);
        if (st != WINDQ_OK) return st;
        hipLaunchKernelGGL(apply_plan_kernel<WINDQ_F32>, grid, dim3(AP_THREADS), lds, hs, A);
    }
    if (hipPeekAtLastError() != hipSuccess) return WINDQ_EHIP;
    return WINDQ_OK;
}
