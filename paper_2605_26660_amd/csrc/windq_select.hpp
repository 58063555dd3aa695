// Rank selection in a histogram, shared by the exact order statistics (P99 of |w| for the
// unit features, the saliency threshold for salient-weight protection).
#pragma once

#include "windq_common.hpp"
#include "windq_ws.hpp"

namespace windq {

// Find, in histogram h of nbins (<= FEAT_BINS) bins, the bin that holds the 1-based `rank`;
// returns the bin and the number of keys in lower bins.  All NT threads of the workgroup call it (NT a multiple of 64 that divides FEAT_BINS).
// Counts fit 32 bits (a unit has fewer than 2^32 weights).  Each thread owns up to 8
// consecutive bins; an exclusive scan over threads (shuffles inside a wavefront, LDS
// across the wavefronts) finds the one thread whose bins straddle the rank.
template <int NT>
__device__ __forceinline__ void select_bin(const uint32_t* __restrict__ h, int nbins, uint64_t rank64,
                                           uint32_t* sh_part, uint32_t* sh_out, uint32_t* bin_out,
                                           uint64_t* below_out) {
    constexpr int PER = FEAT_BINS / NT;
    const uint32_t rank = (uint32_t)rank64;
    const int b0 = threadIdx.x * PER;
    uint32_t v[PER];
    uint32_t local = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        v[j] = b0 + j < nbins ? h[b0 + j] : 0u;
        local += v[j];
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = local;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(inc, d, 64);
        if (lane >= d) inc += t;
    }
    __syncthreads();
    if (lane == 63) sh_part[wave] = inc;
    __syncthreads();
    uint32_t excl = inc - local;
    for (int w = 0; w < wave; ++w) excl += sh_part[w];
    if (excl < rank && rank <= excl + local) {
        uint32_t cum = excl;
        int bin = b0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            if (cum < rank && rank <= cum + v[j]) {
                bin = b0 + j;
                break;
            }
            cum += v[j];
        }
        sh_out[0] = (uint32_t)bin;
        sh_out[1] = cum;
    }
    __syncthreads();
    *bin_out = sh_out[0];
    *below_out = (uint64_t)sh_out[1];
}


}  // namespace windq
