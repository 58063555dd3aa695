// windq_unit_features: the tensor-statistics part of the controller's state (Table 1):
// dims 0-4 (mean, std, mean|w|, fraction |w| < 1e-6, fraction |w| > 0.5 P99) for every
// unit, and dims 9-11 (mean, std, max of the activation scale over the unit's chunk).
//
// Everything but P99 is a streaming reduction (fp64 sums, integer counts), bound by HBM.
// P99 is the exact nearest-rank order statistic of |w|, found by most-significant-digit
// radix selection on the bit pattern of |w| (monotone in |w| for non-negative floats).
//
// The FIRST pass over W -- moments, the count of |w| < 1e-6 and the histograms -- is made by
// the tile kernel of fit_score.hip: either alone (windq_unit_features) or as part of the
// fit+score kernel, which has the tile in LDS anyway (windq_features_fit_score: W is then read
// once for both).  This file holds what follows.
// bf16 (15-bit keys, digits of 11 + 4 bits): NO further pass over W.  The tile kernel counts
//   its tile key by key in LDS, adds the first-digit sums to the unit's histogram, and records
//   the full-resolution counts of 64 first-digit bins (8 octaves: 3 below to 5 above the
//   tile's mean |w|) together with the bin of its largest key.
//   finish  per unit: the first-digit bin e0 of the rank; the 16 + 16 full-resolution counters
//           of e0 and of the bin that holds the key of 0.5*P99, gathered from the unit's tiles'
//           records (a tile whose largest key lies below a bin holds nothing in it).  Halving a
//           bf16 lowers its key by 128 (one exponent step), so that bin is e0 - 8 whatever the
//           low bits of P99 turn out to be.  Then P99 exactly, the exact count of
//           |w| > 0.5 P99 = (first-digit bins above) + (refined counters above), and the eight
//           features.
//   exact   a unit whose bins lie outside the record of one of its tiles (P99 or its half
//           far from 1.6-3.2 times that tile's mean |w|), or whose P99 lies outside the range the tile kernel
//           resolves (below 2^-20 or above 13.5), is counted and listed (for the caller to ask about),
//           and the workgroup that finishes it goes on to select P99 by two digit passes over the
//           unit's weights and to count in a third.  W is read only for such units.
// fp32 (31-bit keys, digits 11 + 11 + 9): one pass per further digit plus a counting pass
// (2|w| > P99, exact in fp32), each re-deriving the prefix from the finished histograms.
// Passes after the first re-read a matrix that was just streamed; up to the 256 MB
// last-level cache they are served on chip.  Integer atomics only, fixed-order fp64
// sums: results are bit-reproducible.
#include <math.h>
#include <string.h>

#include "windq_common.hpp"
#include "windq_feat.hpp"
#include "windq_select.hpp"
#include "windq_ws.hpp"

namespace windq {

constexpr int FT_THREADS = 256;
constexpr int FT_WAVES = FT_THREADS / 64;
constexpr int FEAT_BATCH = 8;   // 128-bit loads a thread keeps in flight

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

// Digit plan: level -> (shift, bits).
template <int DT>
__device__ __host__ constexpr int level_shift(int level) {
    return DT == WINDQ_BF16 ? (level == 0 ? 4 : 0) : (level == 0 ? 20 : (level == 1 ? 9 : 0));
}
template <int DT>
__device__ __host__ constexpr int level_bits(int level) {
    return DT == WINDQ_BF16 ? (level == 0 ? 11 : 4) : (level == 2 ? 9 : 11);
}
template <int DT>
__device__ __host__ constexpr int n_levels() { return DT == WINDQ_BF16 ? 2 : 3; }

// Counters the passes add to: bf16, the first-digit histogram of every unit (and the length of
// the list of units for the exact pass); fp32, all three histograms.
template <int DT>
__host__ __device__ constexpr int64_t feat_init_per_unit() { return DT == WINDQ_BF16 ? FEAT_BINS : 3 * FEAT_BINS; }

template <int DT>
__global__ __launch_bounds__(256) void feat_init_kernel(const FeatBatch B) {
    const int mi = batch_index(B.init_start, B.n, blockIdx.x);
    const FeatArgs& A = B.m[mi];
    const int64_t i = ((int64_t)blockIdx.x - B.init_start[mi]) * 256 + threadIdx.x;
    if (i < feat_init_per_unit<DT>() * A.g.U) A.hist[i] = 0;
    if (DT == WINDQ_BF16 && i == 0) *A.list_count = 0u;
}

// Block-wide sum of a per-thread double in a fixed order (lanes by butterfly, wavefronts in order).
__device__ __forceinline__ double block_sum(double v, double* red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < FT_WAVES; ++w) t += red[w];
    return t;
}

// Key prefix of the wanted rank after digits 0 .. upto-1, from the finished histograms of
// unit u, and the rank still to find under that prefix.
template <int DT>
__device__ __forceinline__ void select_prefix(const FeatArgs& A, int64_t u, int upto, uint32_t* sh_part,
                                              uint32_t* sh_out, uint32_t* prefix_out, uint64_t* rank_out) {
    uint32_t prefix = 0;
    uint64_t rank = A.rank;
    for (int l = 0; l < upto; ++l) {
        const uint32_t* h = A.hist + ((size_t)l * (size_t)A.g.U + (size_t)u) * FEAT_BINS;
        uint32_t bin;
        uint64_t below;
        select_bin<FT_THREADS>(h, 1 << level_bits<DT>(l), rank, sh_part, sh_out, &bin, &below);
        prefix = (prefix << level_bits<DT>(l)) | bin;
        rank -= below;
    }
    *prefix_out = prefix;
    *rank_out = rank;
}

// bf16: first-digit bin that holds the key of 0.5 * P99, given P99's first-digit bin.
__device__ __forceinline__ uint32_t half_bin_of(uint32_t e0) { return e0 >= 16u ? e0 - 8u : e0 >> 1; }

// One pass over FEAT_TPB tiles of one unit (generic element type; used for fp32 inputs).
//   MODE 1: histogram(s) of digit `level` under the unit's prefix.
//   MODE 2: fp32 only: count 2|w| > P99.
template <int DT, int MODE>
__global__ __launch_bounds__(FT_THREADS) void feat_pass_kernel(const FeatBatch B, const int32_t level) {
    __shared__ uint32_t lhist[FEAT_BINS];
    __shared__ double red[FT_WAVES];
    __shared__ uint32_t sh_part[FT_THREADS];
    __shared__ uint32_t sh_out[4];
    const int mi = batch_index(B.block_start, B.n, blockIdx.x);
    const FeatArgs& A = B.m[mi];
    const int64_t wg = (int64_t)blockIdx.x - B.block_start[mi];
    const int64_t u = wg / A.bpu;
    const int64_t blk = wg - u * A.bpu;
    const int32_t G = A.g.chunk_w;
    const int32_t pieces = G >> 3;
    const int64_t rb = u / A.g.n_chunks;
    const int64_t col0 = (u - rb * A.g.n_chunks) * G;
    const int64_t lrow0 = blk * FEAT_TPB * TILE_ROWS;
    const int64_t left = A.g.R_u - lrow0;
    const int32_t nrows = (int32_t)(left < FEAT_TPB * TILE_ROWS ? left : FEAT_TPB * TILE_ROWS);
    const int64_t row0 = rb * A.g.R_u + lrow0;
    const int32_t total = nrows * pieces;
    const int32_t shift = MODE == 2 ? 0 : level_shift<DT>(level);
    const int32_t bits = MODE == 2 ? 0 : level_bits<DT>(level);
    const int32_t nbins = MODE == 2 ? 0 : (DT == WINDQ_BF16 && MODE == 1 ? 32 : (1 << bits));
    const uint32_t mask = (1u << bits) - 1u;
    if (MODE != 2) {
        for (int32_t b = threadIdx.x; b < nbins; b += FT_THREADS) lhist[b] = 0;
    }
    uint32_t prefix = 0, half_bin = 0;
    uint64_t rank_left = 0;
    float p99 = 0.0f;
    if (MODE == 1) {
        select_prefix<DT>(A, u, level, sh_part, sh_out, &prefix, &rank_left);
        half_bin = half_bin_of(prefix);
    }
    if (MODE == 2) {
        select_prefix<DT>(A, u, n_levels<DT>(), sh_part, sh_out, &prefix, &rank_left);
        p99 = value_of_key<DT>(prefix);
    }
    __syncthreads();

    uint32_t cnt = 0;
    auto consume = [&](const float (&w)[8]) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float aw = fabsf(w[j]);
            if (MODE == 1) {
                const uint32_t key = key_of<DT>(w[j]);
                if (DT == WINDQ_BF16) {
                    const uint32_t b = key >> 4;
                    if (b == prefix || b == half_bin) atomicAdd(&lhist[(b == prefix ? 0u : 16u) + (key & 15u)], 1u);
                } else {
                    if ((key >> (shift + bits)) == prefix) atomicAdd(&lhist[(key >> shift) & mask], 1u);
                }
            } else {
                cnt += 2.0f * aw > p99 ? 1u : 0u;
            }
        }
    };
    // Each thread keeps FEAT_BATCH independent 128-bit loads in flight.  When the pieces of
    // a row divide the workgroup, a thread keeps its column piece and steps down the rows
    // (no division per piece); otherwise pieces are dealt out linearly.
    if (FT_THREADS % pieces == 0) {
        const int32_t rstep = FT_THREADS / pieces;
        const int32_t pc = threadIdx.x % pieces;
        const int64_t cbase = col0 + (int64_t)pc * 8;
        for (int32_t r = threadIdx.x / pieces; r < nrows; r += FEAT_BATCH * rstep) {
            float w[FEAT_BATCH][8];
#pragma unroll
            for (int b = 0; b < FEAT_BATCH; ++b)
                if (r + b * rstep < nrows) load8<DT>(A.W, (row0 + r + b * rstep) * A.g.ld + cbase, w[b]);
#pragma unroll
            for (int b = 0; b < FEAT_BATCH; ++b)
                if (r + b * rstep < nrows) consume(w[b]);
        }
    } else {
        for (int32_t i = threadIdx.x; i < total; i += FT_THREADS) {
            const int32_t r = i / pieces;
            const int32_t pc = i - r * pieces;
            float w[8];
            load8<DT>(A.W, (row0 + r) * A.g.ld + col0 + (int64_t)pc * 8, w);
            consume(w);
        }
    }

    const size_t slot = (size_t)u * (size_t)A.bpu + (size_t)blk;
    if (MODE == 2) {
        const double r3 = block_sum((double)cnt, red);
        if (threadIdx.x == 0) A.above[slot] = (uint32_t)r3;
    }
    if (MODE != 2) {
        __syncthreads();
        uint32_t* __restrict__ gh = A.hist + ((size_t)level * (size_t)A.g.U + (size_t)u) * FEAT_BINS;
        for (int32_t b = threadIdx.x; b < nbins; b += FT_THREADS) {
            const uint32_t v = lhist[b];
            if (v != 0) atomicAdd(&gh[b], v);
        }
    }
}

// Block-wide sums of N per-thread doubles at once (one pair of barriers), each in the fixed
// order of block_sum.
template <int N>
__device__ __forceinline__ void block_sum_n(double (&v)[N], double* red) {
#pragma unroll
    for (int j = 0; j < N; ++j) v[j] = wave_sum(v[j]);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int j = 0; j < N; ++j) red[j * FT_WAVES + (threadIdx.x >> 6)] = v[j];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < N; ++j) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < FT_WAVES; ++w) t += red[j * FT_WAVES + w];
        v[j] = t;
    }
}

// bf16: a unit whose P99 the tiles' records do not decide, by the workgroup that finishes it.  P99 by
// two digit passes over the unit's keys (8 + 7 bits), then the count of keys above the key of
// 0.5 * P99: feature 4, the only one that depends on P99.  Called by all threads of the workgroup.
__device__ __forceinline__ void feat_exact_bf16_unit(const FeatArgs& A, int64_t u, uint32_t* h, uint32_t* sh_part,
                                                     uint32_t* sh_out, uint32_t* wsum) {
    static_assert(FT_THREADS == 256, "one thread per bin of the first digit");
    const int tid = threadIdx.x;
    const int32_t G = A.g.chunk_w;
    const int32_t pieces = G >> 3;
    const int64_t total = A.g.R_u * pieces;
    const uint16_t* __restrict__ Wp = static_cast<const uint16_t*>(A.W);
    const int64_t rb = u / A.g.n_chunks;
    const int64_t col0 = (u - rb * A.g.n_chunks) * G;
    const int64_t row0 = rb * A.g.R_u;
    // calls f(key) for every weight of the unit
    auto sweep = [&](auto f) {
        for (int64_t i = tid; i < total; i += FT_THREADS) {
            const int64_t r = i / pieces;
            const int64_t pc = i - r * pieces;
            const uint4 raw = *reinterpret_cast<const uint4*>(Wp + (row0 + r) * A.g.ld + col0 + pc * 8);
            const uint32_t x[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f(x[j] & 0x7fffu);
                f((x[j] >> 16) & 0x7fffu);
            }
        }
    };
    __syncthreads();
    h[tid] = 0u;
    __syncthreads();
    sweep([&](uint32_t key) { atomicAdd(&h[key >> 7], 1u); });
    __syncthreads();
    uint32_t d0, d1;
    uint64_t below;
    select_bin<FT_THREADS>(h, 256, A.rank, sh_part, sh_out, &d0, &below);
    const uint64_t rank1 = A.rank - below;
    __syncthreads();
    h[tid] = 0u;
    __syncthreads();
    sweep([&](uint32_t key) {
        if ((key >> 7) == d0) atomicAdd(&h[key & 127u], 1u);
    });
    __syncthreads();
    select_bin<FT_THREADS>(h, 128, rank1, sh_part, sh_out, &d1, &below);
    // Key of 0.5 * P99: one exponent step down, or half the key where keys are linear in
    // the value (below 256: subnormals and the first binade).
    const uint32_t pk = (d0 << 7) | d1;
    const uint32_t tk = pk >= 256u ? pk - 128u : pk >> 1;
    uint32_t cnt = 0;
    sweep([&](uint32_t key) { cnt += key > tk ? 1u : 0u; });
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) cnt += __shfl_xor(cnt, m, 64);
    __syncthreads();
    if ((tid & 63) == 0) wsum[tid >> 6] = cnt;
    __syncthreads();
    if (tid == 0) {
        uint64_t above = 0;
        for (int w = 0; w < FT_WAVES; ++w) above += wsum[w];
        A.feat[u * WINDQ_N_FEAT + 4] = (float)((double)above / ((double)A.g.R_u * (double)G));
    }
}

// Per unit: P99's key from the finished histograms, the count above half of it, the
// moments in block order, the statistics of s over the chunk; writes the eight features.
// The kernel is a chain of memory latencies (32-86 workgroups, nothing to overlap them
// with), so everything the selection does not decide is requested before it starts: the
// first round of block moments, the activation scales and the refined counters travel
// together with the first-digit histogram.
template <int DT>
__global__ __launch_bounds__(FT_THREADS) void feat_finish_kernel(const FeatBatch B) {
    __shared__ double red[6 * FT_WAVES];
    __shared__ uint32_t sh_part[FT_THREADS];
    __shared__ uint32_t sh_out[4];
    __shared__ float smax_sh[FT_THREADS];
    const int mi = batch_index(B.unit_start, B.n, blockIdx.x);
    const FeatArgs& A = B.m[mi];
    const int64_t u = (int64_t)blockIdx.x - B.unit_start[mi];
    const int32_t G = A.g.chunk_w;
    const float* __restrict__ sc = A.s + (u % A.g.n_chunks) * G;
    const int tid = threadIdx.x;
    // requested now, used after the selection
    static_assert(WINDQ_MAX_CHUNK <= 2 * FT_THREADS, "two activation scales per thread cover a chunk");
    double mv[4] = {0.0, 0.0, 0.0, 0.0};
    if (tid < A.mparts) {
        const double* src = A.moments + ((size_t)u * (size_t)A.mparts + (size_t)tid) * 4;
        mv[0] = src[0]; mv[1] = src[1]; mv[2] = src[2]; mv[3] = src[3];
    }
    const bool has0 = tid < G, has1 = tid + FT_THREADS < G;
    const float sv0 = has0 ? sc[tid] : 0.0f;
    const float sv1 = has1 ? sc[tid + FT_THREADS] : 0.0f;
    const uint32_t* h0 = A.hist + (size_t)u * FEAT_BINS;

    double above = 0.0;
    bool listed = false;        // bf16: left to the exact pass
    if (DT == WINDQ_BF16) {
        __shared__ uint32_t sub[32];          // full-resolution counters of bins e0 and e0 - 8
        __shared__ uint32_t tcnt[FT_THREADS * 33];
        __shared__ int miss;
        uint32_t e0, l1;
        uint64_t rank1, below;
        if (tid == 0) miss = 0;
        // (requested ahead of the selection, like the moments: where this thread's first tile's record lies)
        const uint32_t an_first = tid < A.g.tiles_per_unit ? A.anchor[(size_t)u * (size_t)A.g.tiles_per_unit + (size_t)tid] : 0u;
        select_prefix<DT>(A, u, 1, sh_part, sh_out, &e0, &rank1);       // (its barriers publish the zero)
        const uint32_t eh = half_bin_of(e0);
        // both bins inside the range the tile kernel resolves key by key?
        const bool resolved = eh > (uint32_t)FEAT_FINE_COARSE0 && e0 < (uint32_t)(FEAT_FINE_COARSE0 + FEAT_FINE_NCOARSE - 1);
        uint32_t cnt[32];                     // this thread's tiles (LDS atomics on 32 shared counters crawl)
#pragma unroll
        for (int k = 0; k < 32; ++k) cnt[k] = 0u;
        if (resolved) {
            for (int64_t t = tid; t < A.g.tiles_per_unit; t += FT_THREADS) {
                const size_t tidx = (size_t)u * (size_t)A.g.tiles_per_unit + (size_t)t;
                const uint32_t an = t == tid ? an_first : A.anchor[tidx];
                const uint32_t ct = an & 0xffffu, tmax = an >> 16;     // record = bins ct - 63 .. ct; nothing above tmax
                const uint32_t* __restrict__ rec = A.fine + tidx * (FEAT_WIN * 8);
#pragma unroll
                for (int which = 0; which < 2; ++which) {
                    const uint32_t c = which == 0 ? e0 : eh;
                    if (c > tmax) continue;
                    if (c > ct || c + (FEAT_WIN - 1) < ct) {           // outside the tile's record
                        miss = 1;
                        continue;
                    }
                    const uint4* __restrict__ src = reinterpret_cast<const uint4*>(rec + (c + (FEAT_WIN - 1) - ct) * 8);
                    const uint4 a = src[0], b = src[1];
                    const uint32_t v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        cnt[which * 16 + 2 * i] += v[i] & 0xffffu;
                        cnt[which * 16 + 2 * i + 1] += v[i] >> 16;
                    }
                }
            }
        }
        // the threads that took tiles lay their counters out in LDS (rows of 33: no bank shared by a
        // column), and thread k adds up column k (a butterfly of 32 x 6 shuffles took several times as long)
        const int nact = A.g.tiles_per_unit < (int64_t)FT_THREADS ? (int)A.g.tiles_per_unit : FT_THREADS;
        if (tid < nact) {
#pragma unroll
            for (int k = 0; k < 32; ++k) tcnt[tid * 33 + k] = cnt[k];
        }
        __syncthreads();
        if (tid < 32) {
            uint32_t v = 0;
            for (int r = 0; r < nact; ++r) v += tcnt[r * 33 + tid];
            sub[tid] = v;
        }
        __syncthreads();
        listed = !resolved || miss != 0;
        if (!listed) {
            select_bin<FT_THREADS>(sub, 16, rank1, sh_part, sh_out, &l1, &below);
            // Key of 0.5 * P99: one exponent step down (the resolved range lies far above the
            // first binade, where keys are linear in the value).
            const uint32_t pk = (e0 << 4) | l1;
            const uint32_t tk = pk - 128u;
            const uint32_t tbin = tk >> 4, tlow = tk & 15u;        // tbin == eh by construction
            for (int32_t b = tid; b < FEAT_BINS; b += FT_THREADS)
                if ((uint32_t)b > tbin) above += (double)h0[b];
            if (tid < 16 && (uint32_t)tid > tlow) above += (double)sub[16 + tid];
        } else if (tid == 0) {
            A.list[atomicAdd(A.list_count, 1u)] = (uint32_t)u;
        }
    } else {
        for (int64_t b = tid; b < A.bpu; b += FT_THREADS) above += (double)A.above[(size_t)u * A.bpu + b];
    }

    double m[4] = {mv[0], mv[1], mv[2], mv[3]};
    for (int64_t b = tid + FT_THREADS; b < A.mparts; b += FT_THREADS) {
        const double* src = A.moments + ((size_t)u * (size_t)A.mparts + (size_t)b) * 4;
        m[0] += src[0]; m[1] += src[1]; m[2] += src[2]; m[3] += src[3];
    }
    double ssum = 0.0;
    float smax = sc[0];
    if (has0) { ssum += (double)sv0; smax = fmaxf(smax, sv0); }
    if (has1) { ssum += (double)sv1; smax = fmaxf(smax, sv1); }
    double r6[6] = {above, m[0], m[1], m[2], m[3], ssum};
    block_sum_n<6>(r6, red);
    smax_sh[tid] = smax;
    const double smean = r6[5] / (double)G;
    double sdev = 0.0;
    if (has0) { const double d = (double)sv0 - smean; sdev = fma(d, d, sdev); }
    if (has1) { const double d = (double)sv1 - smean; sdev = fma(d, d, sdev); }
    sdev = block_sum(sdev, red);   // its barriers also publish smax_sh
    if (tid == 0) {
        float mx = smax_sh[0];
        for (int i = 1; i < FT_THREADS; ++i) mx = fmaxf(mx, smax_sh[i]);
        const double n = (double)A.g.R_u * (double)G;
        const double mean = r6[1] / n;
        double var = r6[2] / n - mean * mean;
        var = var > 0.0 ? var : 0.0;
        float* f = A.feat + u * WINDQ_N_FEAT;
        f[0] = (float)mean;
        f[1] = (float)sqrt(var);
        f[2] = (float)(r6[3] / n);
        f[3] = (float)(r6[4] / n);
        if (!listed) f[4] = (float)(r6[0] / n);
        f[5] = (float)smean;
        f[6] = (float)sqrt(sdev / (double)G);
        f[7] = mx;
    }
    if (DT == WINDQ_BF16 && listed) {          // (the same decision in every thread)
        __shared__ uint32_t xh[256];
        __shared__ uint32_t xsum[FT_WAVES];
        feat_exact_bf16_unit(A, u, xh, sh_part, sh_out, xsum);
    }
}

template <int DT>
static int launch_rest(const FeatBatch& B, hipStream_t hs) {
    if (DT == WINDQ_BF16) {
        hipLaunchKernelGGL((feat_finish_kernel<DT>), dim3((unsigned)B.units_total), dim3(FT_THREADS), 0, hs, B);
    } else {
        const dim3 blocks((unsigned)B.blocks_total);
        hipLaunchKernelGGL((feat_pass_kernel<DT, 1>), blocks, dim3(FT_THREADS), 0, hs, B, 1);
        hipLaunchKernelGGL((feat_pass_kernel<DT, 1>), blocks, dim3(FT_THREADS), 0, hs, B, 2);
        hipLaunchKernelGGL((feat_pass_kernel<DT, 2>), blocks, dim3(FT_THREADS), 0, hs, B, 0);
        hipLaunchKernelGGL((feat_finish_kernel<DT>), dim3((unsigned)B.units_total), dim3(FT_THREADS), 0, hs, B);
    }
    return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
}

int features_launch_init(const FeatBatch& B, hipStream_t hs) {
    if (B.dtype == WINDQ_BF16) hipLaunchKernelGGL(feat_init_kernel<WINDQ_BF16>, dim3((unsigned)B.init_total), dim3(256), 0, hs, B);
    else hipLaunchKernelGGL(feat_init_kernel<WINDQ_F32>, dim3((unsigned)B.init_total), dim3(256), 0, hs, B);
    return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
}

int features_launch_rest(const FeatBatch& B, hipStream_t hs) {
    return B.dtype == WINDQ_BF16 ? launch_rest<WINDQ_BF16>(B, hs) : launch_rest<WINDQ_F32>(B, hs);
}

int features_fill(const FeatItem* items, int32_t n, int32_t chunk_w, int64_t unit_rows, FeatBatch* Bp) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    FeatBatch& B = *Bp;
    B.n = n;
    int64_t blocks = 0, units = 0, inits = 0;
    float thr = (float)1e-6;
    if ((double)thr < 1e-6) thr = nextafterf(thr, INFINITY);
    // bf16 keys order like their values: the smallest key whose value reaches the threshold
    uint32_t thr_bits;
    memcpy(&thr_bits, &thr, sizeof thr_bits);
    const uint32_t sparse_key = (thr_bits >> 16) + ((thr_bits & 0xffffu) != 0u ? 1u : 0u);
    static_assert(FEAT_FINE_COARSE0 == 847 && FEAT_FINE_NCOARSE == 200, "1e-6 lies inside the range the tile kernel resolves");
    for (int32_t i = 0; i < n; ++i) {
        const FeatItem& it = items[i];
        FeatArgs& A = B.m[i];
        if (it.W == nullptr) return WINDQ_EINVAL;
        const int st = make_geometry(it.W, chunk_w, unit_rows, &A.g);
        if (st != WINDQ_OK) return st;
        if (it.s == nullptr || it.feat == nullptr) return WINDQ_EINVAL;
        if (it.W->dtype != items[0].W->dtype) return WINDQ_EINVAL;        // one kernel per launch
        const FeatLayout L = features_layout(A.g, it.W->dtype);
        if (it.ws == nullptr || it.ws_bytes < L.total || !aligned(it.ws, 256)) return WINDQ_EWORKSPACE;
        if ((uint64_t)A.g.R_u * (uint64_t)chunk_w > (uint64_t)0xffffffffu) return WINDQ_ESHAPE;   // u32 bin counts
        char* base = static_cast<char*>(it.ws);
        A.W = it.W->data;
        A.s = it.s;
        A.feat = it.feat;
        A.moments = reinterpret_cast<double*>(base + L.moments);
        A.above = reinterpret_cast<uint32_t*>(base + L.above);
        A.hist = reinterpret_cast<uint32_t*>(base + L.hist);
        A.fine = reinterpret_cast<uint32_t*>(base + L.fine);
        A.anchor = reinterpret_cast<uint32_t*>(base + L.anchor);
        A.list_count = reinterpret_cast<uint32_t*>(base + L.list_count);
        A.list = reinterpret_cast<uint32_t*>(base + L.list);
        A.sparse_key = sparse_key;
        A.bpu = L.bpu;
        A.mparts = L.mparts;
        A.sparse_thr = thr;
        const uint64_t nw = (uint64_t)A.g.R_u * (uint64_t)chunk_w;
        A.rank = (99 * nw + 99) / 100;
        B.block_start[i] = blocks;
        B.unit_start[i] = units;
        B.init_start[i] = inits;
        blocks += L.n_blocks;
        units += A.g.U;
        inits += ((items[0].W->dtype == WINDQ_BF16 ? feat_init_per_unit<WINDQ_BF16>() : feat_init_per_unit<WINDQ_F32>()) * A.g.U + 255) / 256;
    }
    for (int32_t i = n; i <= WINDQ_MAX_BATCH; ++i) {
        B.block_start[i] = blocks;
        B.unit_start[i] = units;
        B.init_start[i] = inits;
    }
    for (int32_t i = n; i < WINDQ_MAX_BATCH; ++i) B.m[i] = B.m[0];
    if (blocks > (int64_t)0x7fffffff || inits > (int64_t)0x7fffffff) return WINDQ_ESHAPE;
    B.dtype = items[0].W->dtype;
    B.blocks_total = blocks;
    B.units_total = units;
    B.init_total = inits;
    return WINDQ_OK;
}

}  // namespace windq

using namespace windq;

static int unit_features_launch(const windq_feat_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows, void* stream) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    FeatItem its[WINDQ_MAX_BATCH];
    for (int32_t i = 0; i < n; ++i) its[i] = {items[i].W, items[i].s, items[i].feat, items[i].ws, items[i].ws_bytes};
    FeatBatch B;
    int st = features_fill(its, n, chunk_w, unit_rows, &B);
    if (st != WINDQ_OK) return st;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    st = features_launch_init(B, hs);
    if (st == WINDQ_OK) st = features_launch_tiles(B, hs);
    if (st == WINDQ_OK) st = features_launch_rest(B, hs);
    return st;
}

extern "C" int windq_unit_features(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows, float* feat,
                                   void* ws, size_t ws_bytes, void* stream) {
    if (W == nullptr) return WINDQ_EINVAL;
    const windq_feat_item it = {W, s, feat, ws, ws_bytes};
    return unit_features_launch(&it, 1, chunk_w, unit_rows, stream);
}

extern "C" int windq_unit_features_batch(const windq_feat_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows,
                                         void* stream) {
    return unit_features_launch(items, n, chunk_w, unit_rows, stream);
}

extern "C" int windq_unit_features_exact_units(const void* ws, int32_t dtype, int64_t rows, int64_t cols, int32_t chunk_w,
                                               int64_t unit_rows, int64_t* n_units) {
    if (ws == nullptr || n_units == nullptr) return WINDQ_EINVAL;
    windq_mat fake = {ws, dtype, 0, rows, cols, cols};      // shape checks only: the data pointer is not read
    Geometry g;
    const int st = make_geometry(&fake, chunk_w, unit_rows, &g);
    if (st != WINDQ_OK) return st;
    *n_units = 0;
    if (dtype != WINDQ_BF16) return WINDQ_OK;
    const FeatLayout L = features_layout(g, dtype);
    uint32_t cnt = 0;
    if (hipMemcpy(&cnt, static_cast<const char*>(ws) + L.list_count, sizeof(cnt), hipMemcpyDeviceToHost) != hipSuccess)
        return WINDQ_EHIP;
    *n_units = (int64_t)cnt;
    return WINDQ_OK;
}
