// Salient-weight protection (Sec. 3.5; App. "Salient Weight Protection"): per unit, the
// n_p = floor(rate * n) weights with the largest saliency |w| * s_c are kept out of the
// low-bit quantizer and stored in INT8; Eq. 5 then charges them 8 bits each.
//
// windq_salient_select  finds the protected set EXACTLY: the saliency threshold T of a
//   unit is the n_p-th largest key, located by most-significant-digit radix selection on
//   the bit pattern of the fp32 saliency (digits of 11 + 11 + 9 bits).  The first digit
//   takes one histogram pass over W (LDS histograms flushed by integer atomics).  Its bin
//   e0 holds well under 1 % of a unit's keys, so a second pass over W writes every mask bit
//   that e0 decides and lists the keys of that bin with their positions; the remaining
//   digits, the ties (weights equal to T are taken in the order of their flat index inside
//   the unit: the first n_p - #above of them) and the listed weights' mask bits are then
//   settled per unit from the list alone.  Units whose bin outgrows the list (a thirty-
//   second of the unit: constant weights, say) take the remaining digits by histogram
//   passes over W instead, count their ties per tile where they are split between kept and
//   protected, and rank them in a last pass.  The result is a bit mask in the layout of W:
//   one byte per 8 columns.
// windq_salient_encode  stores the protected weights: per unit one symmetric scale
//   sigma = fp32(max|w_p| / 127), codes clamp(rne(w * fp32(1/sigma)), -127, 127) in
//   flat-index order, and the activation-weighted error of that INT8 part.
// Everything is integer or fixed-order fp64: bit-reproducible.  Select streams W twice (the
// units that fall back: four times, and a fifth for the tiles of those whose ties are split);
// encode reads the mask twice and of W only the protected elements.  Every kernel takes a
// batch of matrices, so a decoder block costs twelve launches for select and four for encode.
// None of this is on the per-step hot path (the mask of a matrix is computed once per
// protection rate).
#include <float.h>

#include "windq_common.hpp"
#include "windq_select.hpp"
#include "windq_ws.hpp"

namespace windq {

constexpr int SAL_THREADS = 256;

struct SalArgs {
    const void* W;
    const float* s;
    uint8_t* mask;          // [rows][mask_ld] bytes
    int64_t mask_ld;
    Geometry g;
    uint32_t* hist;         // [3][U][FEAT_BINS]
    uint32_t* prefix;       // [U]  key prefix found so far; after the last digit: the threshold T
    uint32_t* rank;         // [U]  1-based ascending rank still to find under the prefix
    uint32_t* cnt;          // [n_tiles][2]  keys above T, keys equal to T
    uint32_t* eq_before;    // [n_tiles]     ties in earlier tiles of the unit
    uint32_t* need;         // [U]  ties to protect
    uint32_t* flag;         // [U]  1: selected by digit passes over W; 0: from the unit's candidate list
    uint32_t* n_flagged;    // how many units are flagged, and ...
    uint32_t* flagged;      // [U]  ... which, in no particular order
    uint32_t* cand_count;   // [U]  candidates listed
    uint2* cand;            // [U][cap]  (key, flat position in the unit) of the keys in the threshold's first-digit bin
    uint32_t cap;
    uint32_t use_list;      // 0: every unit takes the digit passes (mask not addressable in whole dwords)
    uint32_t n_p;           // protected weights per unit
    uint32_t rank0;         // ascending rank of T: n - n_p + 1
    // encode
    int8_t* prot_codes;     // [U][n_p]
    float* prot_scale;      // [U]
    float* err_prot;        // [U]
    float* tile_max;        // [n_tiles]
    uint32_t* row_off;      // [U * R_u]  protected weights in earlier rows of the unit
    double* err_part;       // [n_tiles]
};

// A launch covers up to WINDQ_MAX_BATCH matrices (one chunk width, one element type): tiles,
// units and the workgroups that clear the histograms are numbered one matrix after the other.
struct SalBatch {
    int32_t n;
    int64_t tile_start[WINDQ_MAX_BATCH + 1];
    int64_t unit_start[WINDQ_MAX_BATCH + 1];
    int64_t fill_start[WINDQ_MAX_BATCH + 1];     // in workgroups of 256 counters
    SalArgs m[WINDQ_MAX_BATCH];
};

__host__ __device__ constexpr int sal_shift(int level) { return level == 0 ? 20 : (level == 1 ? 9 : 0); }
__host__ __device__ constexpr int sal_bits(int level) { return level == 2 ? 9 : 11; }

// Saliency key: the bit pattern of fp32(|w| * |s_c|), one correctly rounded multiply.
// Non-negative floats order like their bit patterns.
__device__ __forceinline__ uint32_t sal_key(float w, float sc) { return __float_as_uint(fabsf(w) * fabsf(sc)); }

template <int DT>
__device__ __forceinline__ void load8g(const void* __restrict__ data, int64_t off, float (&w)[8]) {
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

// The same eight weights in two steps: the raw bytes (4 or 8 registers), then the values.
template <int DT>
struct Raw8 {
    uint4 a, b;
};
template <>
struct Raw8<WINDQ_BF16> {
    uint4 a;
};
template <int DT>
__device__ __forceinline__ Raw8<DT> load8raw(const void* __restrict__ data, int64_t off) {
    Raw8<DT> r;
    if constexpr (DT == WINDQ_BF16) {
        r.a = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(data) + off);
    } else {
        const uint4* src = reinterpret_cast<const uint4*>(static_cast<const float*>(data) + off);
        r.a = src[0];
        r.b = src[1];
    }
    return r;
}
template <int DT>
__device__ __forceinline__ void unpack8raw(const Raw8<DT>& r, float (&w)[8]) {
    if constexpr (DT == WINDQ_BF16) {
        w[0] = bf16_bits_to_f32(r.a.x & 0xffffu); w[1] = __uint_as_float(r.a.x & 0xffff0000u);
        w[2] = bf16_bits_to_f32(r.a.y & 0xffffu); w[3] = __uint_as_float(r.a.y & 0xffff0000u);
        w[4] = bf16_bits_to_f32(r.a.z & 0xffffu); w[5] = __uint_as_float(r.a.z & 0xffff0000u);
        w[6] = bf16_bits_to_f32(r.a.w & 0xffffu); w[7] = __uint_as_float(r.a.w & 0xffff0000u);
    } else {
        w[0] = __uint_as_float(r.a.x); w[1] = __uint_as_float(r.a.y); w[2] = __uint_as_float(r.a.z); w[3] = __uint_as_float(r.a.w);
        w[4] = __uint_as_float(r.b.x); w[5] = __uint_as_float(r.b.y); w[6] = __uint_as_float(r.b.z); w[7] = __uint_as_float(r.b.w);
    }
}

// Weight j (0..7, a run-time index) of the eight.
template <int DT>
__device__ __forceinline__ float raw_elem(const Raw8<DT>& r, int j) {
    if constexpr (DT == WINDQ_BF16) {
        const int d = j >> 1;
        const uint32_t dw = d == 0 ? r.a.x : (d == 1 ? r.a.y : (d == 2 ? r.a.z : r.a.w));
        return __uint_as_float((j & 1) != 0 ? dw & 0xffff0000u : dw << 16);
    } else {
        const int d = j & 3;
        const uint4& q = j < 4 ? r.a : r.b;
        return __uint_as_float(d == 0 ? q.x : (d == 1 ? q.y : (d == 2 ? q.z : q.w)));
    }
}

// One element of W.
template <int DT>
__device__ __forceinline__ float load1g(const void* __restrict__ data, int64_t off) {
    if (DT == WINDQ_BF16) return bf16_bits_to_f32(static_cast<const uint16_t*>(data)[off]);
    return static_cast<const float*>(data)[off];
}

// Zeroes the digit histograms of every matrix of the launch.
__global__ __launch_bounds__(256) void sal_clear_hist_kernel(const SalBatch B) {
    const int mi = batch_index(B.fill_start, B.n, blockIdx.x);
    const SalArgs& A = B.m[mi];
    const int64_t i = ((int64_t)blockIdx.x - B.fill_start[mi]) * 256 + threadIdx.x;
    if (i < (int64_t)3 * A.g.U * FEAT_BINS) A.hist[i] = 0u;
    if (i == 0) *A.n_flagged = 0u;
}

// Clears the mask of a matrix (rows x mask_ld bytes, dense).
__global__ __launch_bounds__(256) void sal_clear_mask_kernel(uint8_t* __restrict__ mask, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) mask[i] = 0;
}

// Block-wide sum of a per-thread u32 (all SAL_THREADS threads call it).
__device__ __forceinline__ uint32_t block_sum_u32(uint32_t v, uint32_t* sh) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t t = 0;
    for (int w = 0; w < SAL_THREADS / 64; ++w) t += sh[w];
    return t;
}

// Histogram of digit `level` of the keys of one tile that carry the unit's prefix.
template <int DT>
__device__ __forceinline__ void sal_hist_tile(const SalArgs& A, const TileCoord& tc, const int level, uint32_t* lhist,
                                              float* scol) {
    const int32_t G = A.g.chunk_w;
    const int32_t nbins = 1 << sal_bits(level);
    for (int32_t b = threadIdx.x; b < nbins; b += SAL_THREADS) lhist[b] = 0;
    for (int32_t c = threadIdx.x; c < G; c += SAL_THREADS) scol[c] = A.s[tc.col0 + c];
    const uint32_t prefix = level == 0 ? 0u : A.prefix[tc.u];
    __syncthreads();
    const int32_t shift = sal_shift(level), bits = sal_bits(level);
    const uint32_t dmask = (1u << bits) - 1u;
    const int32_t pieces = G >> 3;
    const int32_t total = tc.nrows * pieces;
    PieceWalk at((int32_t)threadIdx.x, SAL_THREADS, pieces);
    for (int32_t i = threadIdx.x; i < total; i += SAL_THREADS, at.next()) {
        const int32_t r = at.r, pc = at.pc;
        float w[8];
        load8g<DT>(A.W, (tc.row0 + r) * A.g.ld + tc.col0 + pc * 8, w);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t key = sal_key(w[j], scol[pc * 8 + j]);
            if (level == 0 || (key >> (shift + bits)) == prefix) atomicAdd(&lhist[(key >> shift) & dmask], 1u);
        }
    }
    __syncthreads();
    uint32_t* __restrict__ gh = A.hist + ((size_t)level * (size_t)A.g.U + (size_t)tc.u) * FEAT_BINS;
    for (int32_t b = threadIdx.x; b < nbins; b += SAL_THREADS) {
        const uint32_t v = lhist[b];
        if (v != 0) atomicAdd(&gh[b], v);
    }
}

// The first digit: every tile of the launch.
template <int DT>
__global__ __launch_bounds__(SAL_THREADS) void sal_hist_kernel(const SalBatch B) {
    __shared__ uint32_t lhist[FEAT_BINS];
    __shared__ float scol[WINDQ_MAX_CHUNK];
    const int mi = batch_index(B.tile_start, B.n, blockIdx.x);
    const SalArgs& A = B.m[mi];
    sal_hist_tile<DT>(A, tile_coord(A.g, (int64_t)blockIdx.x - B.tile_start[mi]), 0, lhist, scol);
}

// Per unit: the bin of digit `level` that holds the wanted rank; extends the prefix.  After the
// last digit the prefix is the threshold T, every key of the bin equals T, and the rank left
// over, r, says that the wanted key is the r-th of those e ties in ascending order: r - 1 of
// them count among the kept weights and need = e - r + 1 among the protected ones.
__global__ __launch_bounds__(SAL_THREADS) void sal_prefix_kernel(const SalBatch B, const int level) {
    __shared__ uint32_t sh_part[SAL_THREADS];
    __shared__ uint32_t sh_out[4];
    const int mi = batch_index(B.unit_start, B.n, blockIdx.x);
    const SalArgs& A = B.m[mi];
    const int64_t u = (int64_t)blockIdx.x - B.unit_start[mi];
    if (level > 0 && A.flag[u] == 0u) return;
    const uint32_t rank = level == 0 ? A.rank0 : A.rank[u];
    const uint32_t prefix = level == 0 ? 0u : A.prefix[u];
    const uint32_t* h = A.hist + ((size_t)level * (size_t)A.g.U + (size_t)u) * FEAT_BINS;
    uint32_t bin;
    uint64_t below;
    select_bin<SAL_THREADS>(h, 1 << sal_bits(level), rank, sh_part, sh_out, &bin, &below);
    if (threadIdx.x == 0) {
        const uint32_t left = rank - (uint32_t)below;
        A.prefix[u] = (prefix << sal_bits(level)) | bin;
        A.rank[u] = left;
        if (level == 2) A.need[u] = h[bin] - left + 1u;
        if (level == 0) {
            // the keys of this bin decide the rest: few enough for the unit's list?
            const bool listed = A.use_list != 0u && h[bin] <= A.cap;
            A.flag[u] = listed ? 0u : 1u;
            A.cand_count[u] = 0u;
            if (!listed) A.flagged[atomicAdd(A.n_flagged, 1u)] = (uint32_t)u;
        }
    }
}

// Which of a unit's ties are protected depends on their order only when some of them are not
// (rank left over above 1); otherwise all are, and nothing has to be counted.
__device__ __forceinline__ bool ties_split(const SalArgs& A, int64_t u) { return A.rank[u] > 1u; }

// Per tile of a unit whose ties are split: how many keys equal the threshold.
template <int DT>
__device__ __forceinline__ void sal_count_tile(const SalArgs& A, const TileCoord& tc, float* scol, uint32_t* sh) {
    if (!ties_split(A, tc.u)) return;
    const int32_t G = A.g.chunk_w;
    for (int32_t c = threadIdx.x; c < G; c += SAL_THREADS) scol[c] = A.s[tc.col0 + c];
    const uint32_t T = A.prefix[tc.u];
    __syncthreads();
    const int32_t pieces = G >> 3;
    const int32_t total = tc.nrows * pieces;
    uint32_t eq = 0;
    PieceWalk at((int32_t)threadIdx.x, SAL_THREADS, pieces);
    for (int32_t i = threadIdx.x; i < total; i += SAL_THREADS, at.next()) {
        const int32_t r = at.r, pc = at.pc;
        float w[8];
        load8g<DT>(A.W, (tc.row0 + r) * A.g.ld + tc.col0 + pc * 8, w);
#pragma unroll
        for (int j = 0; j < 8; ++j) eq += sal_key(w[j], scol[pc * 8 + j]) == T ? 1u : 0u;
    }
    eq = block_sum_u32(eq, sh);
    if (threadIdx.x == 0) A.cnt[(size_t)tc.u * (size_t)A.g.tiles_per_unit + (size_t)tc.t] = eq;
}

// Exclusive prefix sum over a workgroup, in thread order (all SAL_THREADS threads call it);
// *total receives the sum.
__device__ __forceinline__ uint32_t block_exclusive_scan_u32(uint32_t v, uint32_t* sh, uint32_t* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(inc, d, 64);
        if (lane >= d) inc += t;
    }
    __syncthreads();
    if (lane == 63) sh[wave] = inc;
    __syncthreads();
    uint32_t excl = inc - v, tot = 0;
    for (int w = 0; w < SAL_THREADS / 64; ++w) {
        if (w < wave) excl += sh[w];
        tot += sh[w];
    }
    *total = tot;
    return excl;
}

// Per unit: ties in earlier tiles (tile order = row order); zeros where the ties are not split.
__global__ __launch_bounds__(SAL_THREADS) void sal_scan_kernel(const SalBatch B) {
    __shared__ uint32_t sh[SAL_THREADS / 64];
    const int mi = batch_index(B.unit_start, B.n, blockIdx.x);
    const SalArgs& A = B.m[mi];
    const int64_t u = (int64_t)blockIdx.x - B.unit_start[mi];
    if (A.flag[u] == 0u) return;
    const int64_t T = A.g.tiles_per_unit;
    const size_t base = (size_t)u * (size_t)T;
    const bool split = ties_split(A, u);
    uint32_t carry = 0;
    for (int64_t t0 = 0; t0 < T; t0 += SAL_THREADS) {
        const int64_t t = t0 + threadIdx.x;
        const uint32_t eq = split && t < T ? A.cnt[base + t] : 0u;
        uint32_t tot;
        const uint32_t excl = block_exclusive_scan_u32(eq, sh, &tot);
        if (t < T) A.eq_before[base + t] = carry + excl;
        carry += tot;
    }
}

// Per tile: the protection bits.  A thread takes eight consecutive columns of a row, i.e. one
// byte of the mask, straight from HBM; threads walk the tile in flat-index order.  Where the
// unit's ties are split, a tie is protected when its rank among the unit's ties, in flat-index
// order, is below `need`: ties in earlier tiles, plus a scan over the workgroup's threads, plus
// the thread's own eight in order.  Elsewhere every tie is protected and nothing is ranked.
template <int DT>
__device__ __forceinline__ void sal_mask_tile(const SalArgs& A, const TileCoord& tc, float* scol, uint32_t* sh) {
    const int32_t G = A.g.chunk_w;
    for (int32_t c = threadIdx.x; c < G; c += SAL_THREADS) scol[c] = A.s[tc.col0 + c];
    const uint32_t T = A.prefix[tc.u];
    const uint32_t need = A.need[tc.u];
    const bool split = ties_split(A, tc.u);
    uint32_t carry = split ? A.eq_before[(size_t)tc.u * (size_t)A.g.tiles_per_unit + (size_t)tc.t] : 0u;
    __syncthreads();
    const int32_t pieces = G >> 3;
    const int32_t total = tc.nrows * pieces;
    PieceWalk at((int32_t)threadIdx.x, SAL_THREADS, pieces);
    for (int32_t i0 = 0; i0 < total; i0 += SAL_THREADS, at.next()) {
        const int32_t i = i0 + threadIdx.x;
        const bool valid = i < total;
        const int32_t r = at.r, pc = at.pc;
        uint32_t key[8];
        uint32_t eq = 0;
        if (valid) {
            float w[8];
            load8g<DT>(A.W, (tc.row0 + r) * A.g.ld + tc.col0 + pc * 8, w);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                key[j] = sal_key(w[j], scol[pc * 8 + j]);
                eq += key[j] == T ? 1u : 0u;
            }
        }
        uint32_t byte = 0;
        if (split) {                                   // uniform over the workgroup
            uint32_t tot;
            uint32_t tie_rank = carry + block_exclusive_scan_u32(eq, sh, &tot);
            carry += tot;
            if (valid) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    bool prot = key[j] > T;
                    if (key[j] == T) {
                        prot = tie_rank < need;
                        ++tie_rank;
                    }
                    byte |= (prot ? 1u : 0u) << j;
                }
            }
        } else if (valid) {
#pragma unroll
            for (int j = 0; j < 8; ++j) byte |= (key[j] >= T ? 1u : 0u) << j;
        }
        if (valid) A.mask[(tc.row0 + r) * A.mask_ld + (tc.col0 >> 3) + pc] = (uint8_t)byte;
    }
}

// The later digits, the tie counts and the masks of the units that do not select from a list: a
// fixed grid walks the tiles of the listed ("flagged") units of every matrix of the launch; with
// none flagged it returns at once.
constexpr int SAL_FLAGGED_GRID = 1024;
constexpr int SAL_WHAT_HIST = 0, SAL_WHAT_COUNT = 1, SAL_WHAT_MASK = 2;
template <int DT, int WHAT>
__global__ __launch_bounds__(SAL_THREADS) void sal_flagged_kernel(const SalBatch B, const int level) {
    __shared__ uint32_t lhist[WHAT == SAL_WHAT_HIST ? FEAT_BINS : 1];
    __shared__ float scol[WINDQ_MAX_CHUNK];
    __shared__ uint32_t sh[SAL_THREADS / 64];
    for (int mi = 0; mi < B.n; ++mi) {
        const SalArgs& A = B.m[mi];
        const int64_t items = (int64_t)*A.n_flagged * A.g.tiles_per_unit;
        for (int64_t it = blockIdx.x; it < items; it += gridDim.x) {
            const int64_t f = it / A.g.tiles_per_unit;
            const TileCoord tc = tile_coord_of_unit(A.g, (int64_t)A.flagged[f], it - f * A.g.tiles_per_unit);
            __syncthreads();        // the previous tile's shared state is no longer read
            if (WHAT == SAL_WHAT_HIST) sal_hist_tile<DT>(A, tc, level, lhist, scol);
            else if (WHAT == SAL_WHAT_COUNT) sal_count_tile<DT>(A, tc, scol, sh);
            else sal_mask_tile<DT>(A, tc, scol, sh);
        }
    }
}

// ------------------------------------------------- selection from the unit's candidate list
// Units whose threshold bin (first digit e0) is small enough -- all but degenerate ones -- need no
// further digit pass over W.  One pass writes the mask bits that e0 already decides (first digit
// above e0: protected; below: not) and lists the keys whose first digit IS e0 with their flat
// position; one workgroup per unit then finds the threshold, and the ties to take, in the list and
// sets the remaining bits.  Two reads of W in all.
constexpr int SAL_CAND_ITERS = 4;       // 16-byte pieces a thread holds at once
template <int DT>
__global__ __launch_bounds__(SAL_THREADS) void sal_cand_kernel(const SalBatch B) {
    __shared__ float scol[WINDQ_MAX_CHUNK];
    __shared__ uint32_t sh[SAL_THREADS / 64];
    __shared__ uint32_t sh_base;
    const int mi = batch_index(B.tile_start, B.n, blockIdx.x);
    const SalArgs& A = B.m[mi];
    const TileCoord tc = tile_coord(A.g, (int64_t)blockIdx.x - B.tile_start[mi]);
    if (A.flag[tc.u] != 0u) return;
    const int32_t G = A.g.chunk_w;
    for (int32_t c = threadIdx.x; c < G; c += SAL_THREADS) scol[c] = A.s[tc.col0 + c];
    const uint32_t e0 = A.prefix[tc.u];
    uint2* __restrict__ list = A.cand + (size_t)tc.u * (size_t)A.cap;
    __syncthreads();
    const int32_t pieces = G >> 3;
    const int32_t total = tc.nrows * pieces;
    PieceWalk walk((int32_t)threadIdx.x, SAL_THREADS, pieces);
    for (int32_t i0 = 0; i0 < total; i0 += SAL_CAND_ITERS * SAL_THREADS) {
        Raw8<DT> raw[SAL_CAND_ITERS];           // kept as loaded: the keys of a candidate piece are formed again
        uint32_t cm[SAL_CAND_ITERS];            // which of a piece's eight keys are candidates
        int32_t rk[SAL_CAND_ITERS], pk[SAL_CAND_ITERS];      // row and piece of each
        uint32_t n_mine = 0;
#pragma unroll
        for (int k = 0; k < SAL_CAND_ITERS; ++k) {
            const int32_t i = i0 + k * SAL_THREADS + (int32_t)threadIdx.x;
            rk[k] = walk.r;
            pk[k] = walk.pc;
            walk.next();
            if (i < total) raw[k] = load8raw<DT>(A.W, (tc.row0 + rk[k]) * A.g.ld + tc.col0 + pk[k] * 8);
        }
#pragma unroll
        for (int k = 0; k < SAL_CAND_ITERS; ++k) {
            const int32_t i = i0 + k * SAL_THREADS + (int32_t)threadIdx.x;
            cm[k] = 0u;
            if (i < total) {
                const int32_t r = rk[k], pc = pk[k];
                float w[8];
                unpack8raw<DT>(raw[k], w);
                uint32_t byte = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t d0 = sal_key(w[j], scol[pc * 8 + j]) >> sal_shift(0);
                    byte |= (d0 > e0 ? 1u : 0u) << j;
                    cm[k] |= (d0 == e0 ? 1u : 0u) << j;
                }
                A.mask[(tc.row0 + r) * A.mask_ld + (tc.col0 >> 3) + pc] = (uint8_t)byte;
                n_mine += (uint32_t)__builtin_popcount(cm[k]);
            }
        }
        // one place in the unit's list for the workgroup's candidates, then each thread's share of it
        // (one atomic per tile: four per tile, one a wavefront, took 2.5 times as long - the answers to
        // atomics on one counter come back one after the other)
        uint32_t tot;
        uint32_t at = block_exclusive_scan_u32(n_mine, sh, &tot);
        if (threadIdx.x == 0) sh_base = tot != 0u ? atomicAdd(&A.cand_count[tc.u], tot) : 0u;
        __syncthreads();
        at += sh_base;
#pragma unroll
        for (int k = 0; k < SAL_CAND_ITERS; ++k) {
            if (cm[k] != 0u) {
                const int32_t r = rk[k], pc = pk[k];
                const uint32_t pos0 = (uint32_t)(tc.lrow0 + r) * (uint32_t)G + (uint32_t)pc * 8u;
                for (uint32_t m = cm[k]; m != 0u; m &= m - 1u) {        // usually one bit
                    const int j = __ffs(m) - 1;
                    if (at < A.cap) list[at] = make_uint2(sal_key(raw_elem<DT>(raw[k], j), scol[pc * 8 + j]), pos0 + (uint32_t)j);
                    ++at;
                }
            }
        }
        __syncthreads();        // sh_base is read before the next round overwrites it
    }
}

// Histogram of `bits` bits at `shift` of field x (0: key, 1: position) of the list's entries that
// satisfy pred, then the bin of 1-based ascending rank `rank`; returns the bin, the count below it
// and the bin's own count.  All SAL_THREADS threads call it.
template <typename Pred>
__device__ __forceinline__ void list_digit(const uint2* __restrict__ list, uint32_t n, int field, int shift, int bits,
                                           uint32_t rank, Pred pred, uint32_t* lh, uint32_t* sh_part, uint32_t* sh_out,
                                           uint32_t* bin, uint32_t* below, uint32_t* in_bin) {
    const int32_t nbins = 1 << bits;
    __syncthreads();
    for (int32_t b = threadIdx.x; b < nbins; b += SAL_THREADS) lh[b] = 0u;
    __syncthreads();
    for (uint32_t i0 = threadIdx.x; i0 < n; i0 += 4 * SAL_THREADS) {       // four loads in flight per thread
        uint2 e[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i0 + k * SAL_THREADS < n) e[k] = list[i0 + k * SAL_THREADS];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i0 + k * SAL_THREADS < n && pred(e[k]))
                atomicAdd(&lh[((field == 0 ? e[k].x : e[k].y) >> shift) & (uint32_t)(nbins - 1)], 1u);
    }
    __syncthreads();
    uint64_t bl;
    select_bin<SAL_THREADS>(lh, nbins, rank, sh_part, sh_out, bin, &bl);
    *below = (uint32_t)bl;
    *in_bin = lh[*bin];
}

// Per unit: the threshold among the listed keys (their first digit is e0; digits of 11 and 9 bits
// remain), the ties to take (by smallest flat position: three digits of the position), and the
// mask bits of every listed weight that is protected.
__global__ __launch_bounds__(SAL_THREADS) void sal_list_kernel(const SalBatch B) {
    __shared__ uint32_t lh[FEAT_BINS];
    __shared__ uint32_t sh_part[SAL_THREADS];
    __shared__ uint32_t sh_out[4];
    const int mi = batch_index(B.unit_start, B.n, blockIdx.x);
    const SalArgs& A = B.m[mi];
    const int64_t u = (int64_t)blockIdx.x - B.unit_start[mi];
    if (A.flag[u] != 0u) return;
    const uint2* __restrict__ list = A.cand + (size_t)u * (size_t)A.cap;
    const uint32_t n = min(A.cand_count[u], A.cap);
    uint32_t b1, b2, below, in_bin;
    list_digit(list, n, 0, sal_shift(1), sal_bits(1), A.rank[u], [](const uint2&) { return true; }, lh, sh_part, sh_out,
               &b1, &below, &in_bin);
    const uint32_t r1 = A.rank[u] - below;
    list_digit(list, n, 0, sal_shift(2), sal_bits(2), r1,
               [=](const uint2& e) { return ((e.x >> sal_shift(1)) & ((1u << sal_bits(1)) - 1u)) == b1; }, lh, sh_part,
               sh_out, &b2, &below, &in_bin);
    const uint32_t T = (A.prefix[u] << (sal_bits(1) + sal_bits(2))) | (b1 << sal_bits(2)) | b2;
    const uint32_t ties = in_bin;
    const uint32_t need = ties - (r1 - below) + 1u;      // the rank left over counts the ties that stay unprotected, plus one
    uint32_t pos_max = 0xffffffffu;                        // ties up to this position are protected
    if (need < ties) {
        // the need-th smallest position among the ties (positions are distinct): digits of 11, 11, 10 bits
        uint32_t p1, p2, p3, bl;
        list_digit(list, n, 1, 21, 11, need, [=](const uint2& e) { return e.x == T; }, lh, sh_part, sh_out, &p1, &bl, &in_bin);
        const uint32_t n1 = need - bl;
        list_digit(list, n, 1, 10, 11, n1, [=](const uint2& e) { return e.x == T && (e.y >> 21) == p1; }, lh, sh_part, sh_out,
                   &p2, &bl, &in_bin);
        const uint32_t n2 = n1 - bl;
        list_digit(list, n, 1, 0, 10, n2, [=](const uint2& e) { return e.x == T && (e.y >> 10) == ((p1 << 11) | p2); }, lh,
                   sh_part, sh_out, &p3, &bl, &in_bin);
        pos_max = (p1 << 21) | (p2 << 10) | p3;
    }
    const int64_t rb = u / A.g.n_chunks;
    const int64_t col0 = (u - rb * A.g.n_chunks) * A.g.chunk_w;
    const uint32_t G = (uint32_t)A.g.chunk_w;
    for (uint32_t i0 = threadIdx.x; i0 < n; i0 += 4 * SAL_THREADS) {
        uint2 e[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i0 + k * SAL_THREADS < n) e[k] = list[i0 + k * SAL_THREADS];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (i0 + k * SAL_THREADS < n && (e[k].x > T || (e[k].x == T && e[k].y <= pos_max))) {
                const uint32_t r = e[k].y / G, c = e[k].y - r * G;
                const int64_t byte = (rb * A.g.R_u + (int64_t)r) * A.mask_ld + ((col0 + (int64_t)c) >> 3);
                atomicOr(reinterpret_cast<uint32_t*>(A.mask + (byte & ~(int64_t)3)),
                         1u << (8u * (uint32_t)(byte & 3) + (c & 7u)));
            }
        }
    }
}

// ---------------------------------------------------------------------------- encode
// The encode kernels stage only the tile's mask bytes (a sixteenth of the weights' bytes at
// bf16) and fetch the few protected weights straight from HBM, one element at a time but
// SAL_GATHER of them in flight per lane: a lane first notes the columns of its next protected
// weights (in LDS: a register array indexed by a running count would live in scratch memory),
// then requests them together, then works through them in column order.
// LDS: [mask tile][s_c of the chunk][SAL_GATHER x 64 column slots].
constexpr int SAL_GATHER = 8;
static size_t sal_gather_lds(int32_t chunk_w);

// Calls f(column, weight) for the protected weights of the lane's row, in column order.
template <int DT, typename F>
__device__ __forceinline__ void for_protected(const void* __restrict__ W, int64_t woff, const uint8_t* __restrict__ mrow,
                                              int32_t G, uint16_t* __restrict__ slots, F f) {
    int32_t c = 0;          // first column of the next mask byte
    uint32_t m = 0;         // bits of the current byte still to take (it covers columns c - 8 .. c - 1)
    for (;;) {
        int n = 0;
        while (n < SAL_GATHER) {
            if (m == 0u) {
                if (c >= G) break;
                m = mrow[c >> 3];
                c += 8;
                continue;
            }
            const int j = __ffs(m) - 1;
            m &= m - 1u;
            slots[n * 64] = (uint16_t)(c - 8 + j);
            ++n;
        }
        if (n == 0) break;
        float w[SAL_GATHER];
        uint32_t col[SAL_GATHER];
#pragma unroll
        for (int k = 0; k < SAL_GATHER; ++k) {
            if (k < n) {
                col[k] = slots[k * 64];
                w[k] = load1g<DT>(W, woff + col[k]);
            }
        }
#pragma unroll
        for (int k = 0; k < SAL_GATHER; ++k)
            if (k < n) f((int32_t)col[k], w[k]);
        if (n < SAL_GATHER) break;       // the row is exhausted
    }
}

// Per tile, one lane per row: protected weights in the row, largest protected magnitude.
template <int DT>
__global__ __launch_bounds__(64) void sal_rows_kernel(const SalBatch B) {
    extern __shared__ char smem[];
    const int mi = batch_index(B.tile_start, B.n, blockIdx.x);
    const SalArgs& A = B.m[mi];
    const TileCoord tc = tile_coord(A.g, (int64_t)blockIdx.x - B.tile_start[mi]);
    const int32_t G = A.g.chunk_w;
    const int lane = threadIdx.x;
    uint8_t* mtile = reinterpret_cast<uint8_t*>(smem);
    uint16_t* slots = reinterpret_cast<uint16_t*>(smem + TILE_ROWS * mask_row_stride(G) + G * sizeof(float)) + lane;
    load_mask_tile(A.mask, A.mask_ld, tc, G, mtile);
    __syncthreads();
    const bool valid = lane < tc.nrows;
    uint32_t n = 0;
    float mx = 0.0f;
    if (valid) {
        const int64_t woff = (tc.row0 + lane) * A.g.ld + tc.col0;
        const uint8_t* mrow = mtile + lane * mask_row_stride(G);
        for_protected<DT>(A.W, woff, mrow, G, slots, [&](int32_t, float w) {
            ++n;
            mx = fmaxf(mx, fabsf(w));
        });
        A.row_off[tc.u * A.g.R_u + tc.lrow0 + lane] = n;
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
    if (lane == 0) A.tile_max[(size_t)tc.u * (size_t)A.g.tiles_per_unit + (size_t)tc.t] = mx;
}

// Per unit: the INT8 scale, and the row counts turned into offsets (exclusive prefix in row order).
__global__ __launch_bounds__(SAL_THREADS) void sal_unit_kernel(const SalBatch B) {
    __shared__ uint32_t sh[SAL_THREADS / 64];
    __shared__ float shm[SAL_THREADS / 64];
    const int mi = batch_index(B.unit_start, B.n, blockIdx.x);
    const SalArgs& A = B.m[mi];
    const int64_t u = (int64_t)blockIdx.x - B.unit_start[mi];
    float mx = 0.0f;
    for (int64_t t = threadIdx.x; t < A.g.tiles_per_unit; t += SAL_THREADS)
        mx = fmaxf(mx, A.tile_max[(size_t)u * (size_t)A.g.tiles_per_unit + (size_t)t]);
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
    if ((threadIdx.x & 63) == 0) shm[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        float m = shm[0];
        for (int w = 1; w < SAL_THREADS / 64; ++w) m = fmaxf(m, shm[w]);
        float sg = m / 127.0f;
        if (!(sg >= FLT_MIN)) sg = 0.0f;
        A.prot_scale[u] = sg;
    }
    // each thread owns a run of consecutive rows: its sum, one scan over the threads, then the
    // run again to write the offsets (one scan per unit instead of one per 256 rows)
    uint32_t* __restrict__ ro = A.row_off + u * A.g.R_u;
    const int64_t run = (A.g.R_u + SAL_THREADS - 1) / SAL_THREADS;
    const int64_t r_lo = (int64_t)threadIdx.x * run;
    const int64_t r_hi = r_lo + run < A.g.R_u ? r_lo + run : A.g.R_u;
    uint32_t mine = 0;
    for (int64_t r = r_lo; r < r_hi; ++r) mine += ro[r];
    uint32_t tot;
    uint32_t pos = block_exclusive_scan_u32(mine, sh, &tot);
    for (int64_t r = r_lo; r < r_hi; ++r) {
        const uint32_t n = ro[r];
        ro[r] = pos;
        pos += n;
    }
}

// Per tile, one lane per row: INT8 codes of the row's protected weights at their place in
// the unit's stream, and the activation-weighted error of the tile's INT8 part.
template <int DT>
__global__ __launch_bounds__(64) void sal_encode_kernel(const SalBatch B) {
    extern __shared__ char smem[];
    const int mi = batch_index(B.tile_start, B.n, blockIdx.x);
    const SalArgs& A = B.m[mi];
    const TileCoord tc = tile_coord(A.g, (int64_t)blockIdx.x - B.tile_start[mi]);
    const int32_t G = A.g.chunk_w;
    const int lane = threadIdx.x;
    uint8_t* mtile = reinterpret_cast<uint8_t*>(smem);
    float* scol = reinterpret_cast<float*>(smem + TILE_ROWS * mask_row_stride(G));
    uint16_t* slots = reinterpret_cast<uint16_t*>(scol + G) + lane;
    load_mask_tile(A.mask, A.mask_ld, tc, G, mtile);
    for (int32_t c = lane; c < G; c += 64) scol[c] = A.s[tc.col0 + c];
    __syncthreads();
    const float sg = A.prot_scale[tc.u];
    const float inv = sg > 0.0f ? 1.0f / sg : 0.0f;
    double err = 0.0;
    if (lane < tc.nrows) {
        const int64_t woff = (tc.row0 + lane) * A.g.ld + tc.col0;
        const uint8_t* mrow = mtile + lane * mask_row_stride(G);
        uint32_t pos = A.row_off[tc.u * A.g.R_u + tc.lrow0 + lane];
        int8_t* __restrict__ dst = A.prot_codes + (size_t)tc.u * (size_t)A.n_p;
        for_protected<DT>(A.W, woff, mrow, G, slots, [&](int32_t c, float w) {
            const float t = w * inv;
            const float q = __builtin_amdgcn_fmed3f(__builtin_rintf(t), -127.0f, 127.0f);
            if (pos < A.n_p) dst[pos] = (int8_t)(int32_t)q;     // a mask with more bits than n_p writes nothing past the unit
            ++pos;
            const double d = (double)w - (double)q * (double)sg;
            const double a = (double)scol[c] * (double)scol[c];
            err = fma(a * d, d, err);
        });
    }
    err = wave_sum(err);
    if (lane == 0) A.err_part[(size_t)tc.u * (size_t)A.g.tiles_per_unit + (size_t)tc.t] = err;
}

__global__ __launch_bounds__(256) void sal_err_kernel(const SalBatch B) {
    __shared__ double red[4];
    const int mi = batch_index(B.unit_start, B.n, blockIdx.x);
    const SalArgs& A = B.m[mi];
    const int64_t u = (int64_t)blockIdx.x - B.unit_start[mi];
    const double e = unit_partial_sum<256>(A.err_part + (size_t)u * (size_t)A.g.tiles_per_unit, A.g.tiles_per_unit, red);
    if (threadIdx.x == 0) A.err_prot[u] = (float)e;
}

// ------------------------------------------------------------------- unit saliency
// Saliency score of a unit (App. "Comparison with Heuristic Sensitivity Allocator"): the mean
// of |w| * |s_c| over the unit.  Per tile an fp64 sum in a fixed order, per unit the tiles in order.
template <int DT>
__global__ __launch_bounds__(SAL_THREADS) void unit_saliency_tile_kernel(const void* __restrict__ W, const float* __restrict__ s,
                                                                         const Geometry g, double* __restrict__ part) {
    __shared__ float scol[WINDQ_MAX_CHUNK];
    __shared__ double red[SAL_THREADS / 64];
    const TileCoord tc = tile_coord(g, blockIdx.x);
    const int32_t G = g.chunk_w;
    for (int32_t c = threadIdx.x; c < G; c += SAL_THREADS) scol[c] = fabsf(s[tc.col0 + c]);
    __syncthreads();
    const int32_t pieces = G >> 3;
    const int32_t total = tc.nrows * pieces;
    double acc = 0.0;
    PieceWalk at((int32_t)threadIdx.x, SAL_THREADS, pieces);
    for (int32_t i = threadIdx.x; i < total; i += SAL_THREADS, at.next()) {
        const int32_t r = at.r, pc = at.pc;
        float w[8];
        load8g<DT>(W, (tc.row0 + r) * g.ld + tc.col0 + pc * 8, w);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc = fma((double)fabsf(w[j]), (double)scol[pc * 8 + j], acc);
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < SAL_THREADS / 64; ++w) t += red[w];
        part[(size_t)tc.u * (size_t)g.tiles_per_unit + (size_t)tc.t] = t;
    }
}

__global__ __launch_bounds__(256) void unit_saliency_finalize_kernel(const double* __restrict__ part, const Geometry g,
                                                                    float* __restrict__ sal) {
    __shared__ double red[4];
    const int64_t u = blockIdx.x;
    const double t = unit_partial_sum<256>(part + (size_t)u * (size_t)g.tiles_per_unit, g.tiles_per_unit, red);
    if (threadIdx.x == 0) sal[u] = (float)(t / ((double)g.R_u * (double)g.chunk_w));
}

// encode's kernels: the tile's mask bytes, s_c of the chunk, the lanes' column slots
static size_t sal_gather_lds(int32_t chunk_w) {
    return mask_tile_lds_bytes(chunk_w) + (size_t)chunk_w * sizeof(float) + (size_t)SAL_GATHER * 64 * sizeof(uint16_t);
}

static void carve(SalArgs& A, void* ws, const SalientLayout& L) {
    char* base = static_cast<char*>(ws);
    A.hist = reinterpret_cast<uint32_t*>(base + L.hist);
    A.prefix = reinterpret_cast<uint32_t*>(base + L.prefix);
    A.rank = reinterpret_cast<uint32_t*>(base + L.rank);
    A.cnt = reinterpret_cast<uint32_t*>(base + L.cnt);
    A.eq_before = reinterpret_cast<uint32_t*>(base + L.eq_before);
    A.need = reinterpret_cast<uint32_t*>(base + L.need);
    A.flag = reinterpret_cast<uint32_t*>(base + L.flag);
    A.n_flagged = reinterpret_cast<uint32_t*>(base + L.n_flagged);
    A.flagged = reinterpret_cast<uint32_t*>(base + L.flagged);
    A.cand_count = reinterpret_cast<uint32_t*>(base + L.cand_count);
    A.cand = reinterpret_cast<uint2*>(base + L.cand);
    A.cap = L.cap;
    A.tile_max = reinterpret_cast<float*>(base + L.tile_max);
    A.row_off = reinterpret_cast<uint32_t*>(base + L.row_off);
    A.err_part = reinterpret_cast<double*>(base + L.err_part);
}

template <int DT>
static int launch_select(const SalBatch& B, hipStream_t hs) {
    const dim3 tiles((unsigned)B.tile_start[B.n]), units((unsigned)B.unit_start[B.n]), some(SAL_FLAGGED_GRID);
    hipLaunchKernelGGL(sal_clear_hist_kernel, dim3((unsigned)B.fill_start[B.n]), dim3(256), 0, hs, B);
    hipLaunchKernelGGL(sal_hist_kernel<DT>, tiles, dim3(SAL_THREADS), 0, hs, B);
    hipLaunchKernelGGL(sal_prefix_kernel, units, dim3(SAL_THREADS), 0, hs, B, 0);
    // units that select from their candidate list ...
    hipLaunchKernelGGL(sal_cand_kernel<DT>, tiles, dim3(SAL_THREADS), 0, hs, B);
    hipLaunchKernelGGL(sal_list_kernel, units, dim3(SAL_THREADS), 0, hs, B);
    // ... and the others
    for (int level = 1; level < 3; ++level) {
        hipLaunchKernelGGL((sal_flagged_kernel<DT, SAL_WHAT_HIST>), some, dim3(SAL_THREADS), 0, hs, B, level);
        hipLaunchKernelGGL(sal_prefix_kernel, units, dim3(SAL_THREADS), 0, hs, B, level);
    }
    hipLaunchKernelGGL((sal_flagged_kernel<DT, SAL_WHAT_COUNT>), some, dim3(SAL_THREADS), 0, hs, B, 0);
    hipLaunchKernelGGL(sal_scan_kernel, units, dim3(SAL_THREADS), 0, hs, B);
    hipLaunchKernelGGL((sal_flagged_kernel<DT, SAL_WHAT_MASK>), some, dim3(SAL_THREADS), 0, hs, B, 0);
    return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
}

template <int DT>
static int launch_encode(const SalBatch& B, hipStream_t hs, size_t lds) {
    const dim3 tiles((unsigned)B.tile_start[B.n]), units((unsigned)B.unit_start[B.n]);
    int st = ensure_lds(reinterpret_cast<const void*>(&sal_rows_kernel<DT>), lds);
    if (st != WINDQ_OK) return st;
    st = ensure_lds(reinterpret_cast<const void*>(&sal_encode_kernel<DT>), lds);
    if (st != WINDQ_OK) return st;
    hipLaunchKernelGGL(sal_rows_kernel<DT>, tiles, dim3(64), lds, hs, B);
    hipLaunchKernelGGL(sal_unit_kernel, units, dim3(SAL_THREADS), 0, hs, B);
    hipLaunchKernelGGL(sal_encode_kernel<DT>, tiles, dim3(64), lds, hs, B);
    hipLaunchKernelGGL(sal_err_kernel, units, dim3(256), 0, hs, B);
    return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
}

}  // namespace windq

using namespace windq;

extern "C" int64_t windq_n_protected(int64_t n_unit, uint32_t rate_ppm) {
    if (n_unit < 0 || rate_ppm > 1000000u) return -1;
    // n * rate fits 64 bits for every n the kernels accept (n < 2^32)
    return (int64_t)(((unsigned __int128)(uint64_t)n_unit * rate_ppm) / 1000000u);
}

static int salient_common(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows, uint32_t rate_ppm,
                          const uint8_t* mask, void* ws, size_t ws_bytes, SalArgs* A) {
    if (W == nullptr) return WINDQ_EINVAL;
    const int st = make_geometry(W, chunk_w, unit_rows, &A->g);
    if (st != WINDQ_OK) return st;
    if (s == nullptr || mask == nullptr || rate_ppm > 1000000u) return WINDQ_EINVAL;
    if ((uint64_t)A->g.R_u * (uint64_t)chunk_w > (uint64_t)0xffffffffu) return WINDQ_ESHAPE;   // u32 counts
    const SalientLayout L = salient_layout(A->g);
    if (ws == nullptr || ws_bytes < L.total || !aligned(ws, 256)) return WINDQ_EWORKSPACE;
    A->W = W->data;
    A->s = s;
    A->mask = const_cast<uint8_t*>(mask);
    A->mask_ld = W->cols / 8;
    const uint64_t n = (uint64_t)A->g.R_u * (uint64_t)chunk_w;
    A->n_p = (uint32_t)windq_n_protected((int64_t)n, rate_ppm);
    A->rank0 = (uint32_t)(n - A->n_p + 1);
    // the list route sets mask bits with 32-bit atomics: the mask has to be addressable in whole dwords
    A->use_list = aligned(mask, 4) && ((uint64_t)W->rows * (uint64_t)A->mask_ld) % 4 == 0 ? 1u : 0u;
    A->prot_codes = nullptr;
    A->prot_scale = nullptr;
    A->err_prot = nullptr;
    carve(*A, ws, L);
    return WINDQ_OK;
}

// Numbers the tiles, units and histogram-clearing workgroups of the first B->n matrices.
static int salient_number(SalBatch* B) {
    int64_t tiles = 0, units = 0, fill = 0;
    for (int32_t i = 0; i < B->n; ++i) {
        B->tile_start[i] = tiles;
        B->unit_start[i] = units;
        B->fill_start[i] = fill;
        tiles += B->m[i].g.n_tiles;
        units += B->m[i].g.U;
        fill += ((int64_t)3 * B->m[i].g.U * FEAT_BINS + 255) / 256;
    }
    for (int32_t i = B->n; i <= WINDQ_MAX_BATCH; ++i) {
        B->tile_start[i] = tiles;
        B->unit_start[i] = units;
        B->fill_start[i] = fill;
    }
    for (int32_t i = B->n; i < WINDQ_MAX_BATCH; ++i) B->m[i] = B->m[0];
    return tiles > (int64_t)0x7fffffff || fill > (int64_t)0x7fffffff ? WINDQ_ESHAPE : WINDQ_OK;
}

static int salient_select_launch(const windq_salient_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows,
                                 uint32_t rate_ppm, void* stream) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    SalBatch B;
    B.n = 0;
    const uint8_t* empty[WINDQ_MAX_BATCH];      // masks of matrices whose units protect nothing
    int64_t empty_bytes[WINDQ_MAX_BATCH];
    int32_t n_empty = 0;
    for (int32_t i = 0; i < n; ++i) {
        SalArgs& A = B.m[B.n];
        const int st = salient_common(items[i].W, items[i].s, chunk_w, unit_rows, rate_ppm, items[i].mask, items[i].ws,
                                      items[i].ws_bytes, &A);
        if (st != WINDQ_OK) return st;
        if (items[i].W->dtype != items[0].W->dtype) return WINDQ_EINVAL;      // one kernel per launch
        if (A.n_p == 0) {
            empty[n_empty] = items[i].mask;
            empty_bytes[n_empty++] = items[i].W->rows * A.mask_ld;
        } else {
            ++B.n;
        }
    }
    hipStream_t hs = static_cast<hipStream_t>(stream);
    for (int32_t i = 0; i < n_empty; ++i)
        hipLaunchKernelGGL(sal_clear_mask_kernel, dim3((unsigned)((empty_bytes[i] + 255) / 256)), dim3(256), 0, hs,
                           const_cast<uint8_t*>(empty[i]), empty_bytes[i]);
    if (B.n == 0) return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
    const int st = salient_number(&B);
    if (st != WINDQ_OK) return st;
    const int32_t dtype = items[0].W->dtype;
    return dtype == WINDQ_BF16 ? launch_select<WINDQ_BF16>(B, hs) : launch_select<WINDQ_F32>(B, hs);
}

static int salient_encode_launch(const windq_salient_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows,
                                 uint32_t rate_ppm, void* stream) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    SalBatch B;
    B.n = n;
    for (int32_t i = 0; i < n; ++i) {
        SalArgs& A = B.m[i];
        const int st = salient_common(items[i].W, items[i].s, chunk_w, unit_rows, rate_ppm, items[i].mask, items[i].ws,
                                      items[i].ws_bytes, &A);
        if (st != WINDQ_OK) return st;
        if (items[i].W->dtype != items[0].W->dtype) return WINDQ_EINVAL;
        if (items[i].prot_scale == nullptr || items[i].err_prot == nullptr) return WINDQ_EINVAL;
        if (items[i].prot_codes == nullptr && A.n_p != 0) return WINDQ_EINVAL;
        A.prot_codes = items[i].prot_codes;
        A.prot_scale = items[i].prot_scale;
        A.err_prot = items[i].err_prot;
    }
    const int st = salient_number(&B);
    if (st != WINDQ_OK) return st;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int32_t dtype = items[0].W->dtype;
    const size_t lds = sal_gather_lds(chunk_w);
    return dtype == WINDQ_BF16 ? launch_encode<WINDQ_BF16>(B, hs, lds) : launch_encode<WINDQ_F32>(B, hs, lds);
}

extern "C" int windq_salient_select(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows,
                                    uint32_t rate_ppm, uint8_t* mask, void* ws, size_t ws_bytes, void* stream) {
    const windq_salient_item it = {W, s, mask, nullptr, nullptr, nullptr, ws, ws_bytes};
    return salient_select_launch(&it, 1, chunk_w, unit_rows, rate_ppm, stream);
}

extern "C" int windq_salient_select_batch(const windq_salient_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows,
                                          uint32_t rate_ppm, void* stream) {
    return salient_select_launch(items, n, chunk_w, unit_rows, rate_ppm, stream);
}

extern "C" int windq_salient_encode(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows,
                                    const uint8_t* mask, uint32_t rate_ppm, int8_t* prot_codes, float* prot_scale,
                                    float* err_prot, void* ws, size_t ws_bytes, void* stream) {
    const windq_salient_item it = {W, s, const_cast<uint8_t*>(mask), prot_codes, prot_scale, err_prot, ws, ws_bytes};
    return salient_encode_launch(&it, 1, chunk_w, unit_rows, rate_ppm, stream);
}

extern "C" int windq_salient_encode_batch(const windq_salient_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows,
                                          uint32_t rate_ppm, void* stream) {
    return salient_encode_launch(items, n, chunk_w, unit_rows, rate_ppm, stream);
}

extern "C" int windq_unit_saliency(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows, float* sal,
                                   void* ws, size_t ws_bytes, void* stream) {
    Geometry g;
    const int st = make_geometry(W, chunk_w, unit_rows, &g);
    if (st != WINDQ_OK) return st;
    if (s == nullptr || sal == nullptr) return WINDQ_EINVAL;
    if (ws == nullptr || ws_bytes < unit_saliency_ws_bytes(g) || !aligned(ws, 256)) return WINDQ_EWORKSPACE;
    double* part = static_cast<double*>(ws);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const dim3 tiles((unsigned)g.n_tiles);
    if (W->dtype == WINDQ_BF16)
        hipLaunchKernelGGL(unit_saliency_tile_kernel<WINDQ_BF16>, tiles, dim3(SAL_THREADS), 0, hs, W->data, s, g, part);
    else
        hipLaunchKernelGGL(unit_saliency_tile_kernel<WINDQ_F32>, tiles, dim3(SAL_THREADS), 0, hs, W->data, s, g, part);
    hipLaunchKernelGGL(unit_saliency_finalize_kernel, dim3((unsigned)g.U), dim3(256), 0, hs, part, g, sal);
    return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
}
