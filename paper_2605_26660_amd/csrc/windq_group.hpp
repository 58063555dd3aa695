// One lane, one group: the normative fp32 quantizers of a row held in LDS (element type of the
// input, see windq_common.hpp), shared by windq_apply_plan and windq_refine_plan.  Packed
// bytes are written back into the row's own LDS storage, behind the read position (b/8 bytes
// per weight never overtake the 2 or 4 bytes read).  `mrow` is the row's protection bits
// (null: none): protected weights stay out of every statistic and their code slot holds 0.
#pragma once

#include <float.h>

#include "windq_common.hpp"

namespace windq {

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

// min and max of the kept weights of a group (0, 0 when none is kept).
template <int DT>
__device__ __forceinline__ void group_min_max(const char* wrow, const uint8_t* __restrict__ mrow, int32_t G, float* mn_out,
                                              float* mx_out) {
    float w[8];
    float mn, mx;
    if (mrow == nullptr) {
        read8<DT>(wrow, 0, w);
        mn = mx = w[0];
        for (int32_t c = 0; c < G; c += 8) {
            read8<DT>(wrow, c, w);
            mn = fminf(fminf(fminf(mn, w[0]), fminf(w[1], w[2])), fminf(fminf(w[3], w[4]), fminf(w[5], fminf(w[6], w[7]))));
            mx = fmaxf(fmaxf(fmaxf(mx, w[0]), fmaxf(w[1], w[2])), fmaxf(fmaxf(w[3], w[4]), fmaxf(w[5], fmaxf(w[6], w[7]))));
        }
    } else {
        mn = INFINITY;
        mx = -INFINITY;
        for (int32_t c = 0; c < G; c += 8) {
            read8<DT>(wrow, c, w);
            const uint32_t m = mrow[c >> 3];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool kept = ((m >> j) & 1u) == 0u;
                mn = fminf(mn, kept ? w[j] : INFINITY);
                mx = fmaxf(mx, kept ? w[j] : -INFINITY);
            }
        }
        if (mn > mx) mn = mx = 0.0f;      // no weight of the group is kept
    }
    *mn_out = mn;
    *mx_out = mx;
}

// Offset and step of the uniform quantizer with qmax + 1 levels at clip ratio p, normative fp32
// steps; a step below the smallest normal fp32 is degenerate (step 0).
__device__ __forceinline__ void uniform_params(float mn, float mx, float p, float qmax, float* lo_out, float* step_out) {
    const float lo = p * mn;
    const float hi = p * mx;
    const float rg = hi - lo;
    float d = rg / qmax;
    d = d >= FLT_MIN ? d : 0.0f;
    *lo_out = lo;
    *step_out = d;
}

// Codes of a group at (lo, step), normative fp32 steps, packed in place.
template <int DT, int BITS>
__device__ __forceinline__ void uniform_pack(const char* wrow, const uint8_t* __restrict__ mrow, int32_t G, float lo, float d,
                                             uint8_t* dst) {
    const float qmax = (float)((1 << BITS) - 1);
    const float inv = d >= FLT_MIN ? 1.0f / d : 0.0f;
    float w[8];
    for (int32_t c = 0; c < G; c += 8) {
        read8<DT>(wrow, c, w);
        const uint32_t m = mrow != nullptr ? mrow[c >> 3] : 0u;     // read before the codes overwrite the row in place
        uint32_t code[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float u = w[j] - lo;
            const float t = u * inv;
            const float q = __builtin_amdgcn_fmed3f(__builtin_rintf(t), 0.0f, qmax);
            code[j] = ((m >> j) & 1u) != 0u ? 0u : (uint32_t)q;
        }
        store_codes8<BITS>(dst + (c >> 3) * BITS, code);
    }
}

// Uniform BITS-bit quantizer of one group: statistics, parameters, codes.
template <int DT, int BITS>
__device__ __forceinline__ void quantize_uniform(const char* wrow, const uint8_t* __restrict__ mrow, int32_t G, float p,
                                                 uint8_t* dst, float* scale_out, float* offset_out) {
    float mn, mx, lo, d;
    group_min_max<DT>(wrow, mrow, G, &mn, &mx);
    uniform_params(mn, mx, p, (float)((1 << BITS) - 1), &lo, &d);
    *scale_out = d;
    *offset_out = lo;
    uniform_pack<DT, BITS>(wrow, mrow, G, lo, d, dst);
}

// Mean |w| of a group as stored: the fp64 sum in column order (exact for bf16 inputs) over the
// kept weights, divided by their number, rounded to fp32; 0 when none is kept.
template <int DT>
__device__ __forceinline__ float group_abs_mean(const char* wrow, const uint8_t* __restrict__ mrow, int32_t G) {
    double S1 = 0.0;
    int32_t n = G;
    for (int32_t c = 0; c < G; c += 8) {
        float w[8];
        read8<DT>(wrow, c, w);
        const uint32_t m = mrow != nullptr ? mrow[c >> 3] : 0u;
        n -= __builtin_popcount(m);
#pragma unroll
        for (int j = 0; j < 8; ++j) S1 += ((m >> j) & 1u) != 0u ? 0.0 : (double)fabsf(w[j]);
    }
    return n > 0 ? (float)(S1 / (double)n) : 0.0f;
}

// Ternary codes of a group at scale gamma (0: degenerate), five trits q + 1 per byte, in place.
template <int DT>
__device__ __forceinline__ void ternary_pack(const char* wrow, const uint8_t* __restrict__ mrow, int32_t G, float gamma,
                                             uint8_t* dst) {
    const float inv = gamma >= FLT_MIN ? 1.0f / gamma : 0.0f;
    uint32_t byte = 0, mul = 1;
    int32_t nb = 0;
    for (int32_t c = 0; c < G; c += 8) {
        float w[8];
        read8<DT>(wrow, c, w);
        const uint32_t m = mrow != nullptr ? mrow[c >> 3] : 0u;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float t = w[j] * inv;
            const float q = __builtin_amdgcn_fmed3f(__builtin_rintf(t), -1.0f, 1.0f);
            byte += (((m >> j) & 1u) != 0u ? 0u : (uint32_t)((int32_t)q + 1)) * mul;
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
__device__ __forceinline__ void quantize_ternary(const char* wrow, const uint8_t* __restrict__ mrow, int32_t G,
                                                 uint8_t* dst, float* scale_out) {
    float gamma = group_abs_mean<DT>(wrow, mrow, G);
    gamma = gamma >= FLT_MIN ? gamma : 0.0f;
    *scale_out = gamma;
    ternary_pack<DT>(wrow, mrow, G, gamma, dst);
}

// Sign bits of a group (w >= 0 -> 1), in place.
template <int DT>
__device__ __forceinline__ void binary_pack(const char* wrow, const uint8_t* __restrict__ mrow, int32_t G, uint8_t* dst) {
    for (int32_t c = 0; c < G; c += 8) {
        float w[8];
        read8<DT>(wrow, c, w);
        const uint32_t m = mrow != nullptr ? mrow[c >> 3] : 0u;
        uint32_t byte = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) byte |= (w[j] >= 0.0f ? 1u : 0u) << j;
        dst[c >> 3] = (uint8_t)(byte & ~m);
    }
}

template <int DT>
__device__ __forceinline__ void quantize_binary(const char* wrow, const uint8_t* __restrict__ mrow, int32_t G,
                                                uint8_t* dst, float* scale_out) {
    *scale_out = group_abs_mean<DT>(wrow, mrow, G);
    binary_pack<DT>(wrow, mrow, G, dst);
}

// Copy a tile's packed rows (bpg bytes each, row_bytes apart in LDS) to one contiguous range
// of the code stream with coalesced stores, in elements of the widest size that divides bpg.
// All `nthreads` threads of the workgroup call it after a barrier.
__device__ __forceinline__ void copy_out_rows(const char* tile, int32_t row_bytes, int32_t bpg, int32_t nrows,
                                              uint8_t* __restrict__ out, int tid, int nthreads) {
    const int32_t e = (bpg & 15) == 0 ? 16 : ((bpg & 3) == 0 ? 4 : ((bpg & 1) == 0 ? 2 : 1));
    const int32_t total = nrows * bpg;
    int32_t byte = tid * e;
    int32_t row = byte / bpg;
    int32_t col = byte - row * bpg;
    for (; byte < total; byte += nthreads * e) {
        const char* src = tile + row * row_bytes + col;
        if (e == 16) *reinterpret_cast<uint4*>(out + byte) = *reinterpret_cast<const uint4*>(src);
        else if (e == 4) *reinterpret_cast<uint32_t*>(out + byte) = *reinterpret_cast<const uint32_t*>(src);
        else if (e == 2) *reinterpret_cast<uint16_t*>(out + byte) = *reinterpret_cast<const uint16_t*>(src);
        else out[byte] = *reinterpret_cast<const uint8_t*>(src);
        col += nthreads * e;
        while (col >= bpg) {
            col -= bpg;
            ++row;
        }
    }
}

}  // namespace windq
