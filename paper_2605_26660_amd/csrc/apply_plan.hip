// windq_apply_plan: materialise a mixed-precision plan as packed codes plus per-group
// scale and offset (Sec. 3.3: the environment applies the selected quantization to the
// unit; Sec. 3.5: the engine applies the operator of the chosen bit-width).
//
// Codes and stored scales are DEFINED by a short sequence of correctly rounded fp32
// operations (see windq.h); this file is compiled with floating-point contraction off so
// that each written operation is exactly one IEEE operation.  The sum of |w| of a group
// is accumulated in fp64 in column order (exact for bf16 inputs).
//
// Streaming kernels, bound by HBM: read 2 (bf16) or 4 (fp32) bytes per weight once,
// write b/8 bytes of codes per weight and 8 bytes per group.  Two kernels: bf16 at chunk
// widths 32/64/128 takes the lanes-per-row kernel further down; everything else takes the
// general kernel described here.  One wavefront per tile of 64 rows x one chunk.  The tile is loaded with coalesced 128-bit loads into LDS in the
// input's own element type (17 KB for bf16 at chunk 128: nine workgroups per CU, whose
// loads overlap each other's arithmetic).  Each lane quantizes and packs its own row, so
// ternary base-3 bytes and 3-bit streams need no cross-lane regrouping, and writes the
// packed bytes back INTO ITS OWN ROW of the tile: packed output never overtakes the read
// position (b/8 <= element bytes).  Rows of a unit are consecutive in the code stream, so
// the 64 packed rows are then copied to one contiguous byte range with coalesced stores.
#include <float.h>

#include <type_traits>

#include "windq_common.hpp"
#include "windq_group.hpp"
#include "windq_ws.hpp"

namespace windq {

constexpr int AP_THREADS = 64;

struct ApplyArgs {
    const void* W;
    const uint8_t* mask;       // protection mask [rows][cols/8] (masked kernel only)
    int64_t mask_ld;
    const uint8_t* action;
    const uint8_t* clip_idx;   // may be null
    const int64_t* code_off;
    uint8_t* codes;
    int64_t codes_bytes;
    float* scale;
    float* offset;
    Geometry g;
};

// A launch covers up to WINDQ_MAX_BATCH matrices (one chunk width, one element type, all with
// or all without a mask): their tiles are numbered one matrix after the other.
struct ApplyBatch {
    int32_t n;
    int32_t K;
    int64_t tile_start[WINDQ_MAX_BATCH + 1];
    ApplyArgs m[WINDQ_MAX_BATCH];
    ClipGrid grid;
};

template <int DT>
__global__ __launch_bounds__(AP_THREADS) void apply_plan_kernel(const ApplyBatch B) {
    extern __shared__ char tile[];
    const int mi = batch_index(B.tile_start, B.n, blockIdx.x);
    const ApplyArgs& A = B.m[mi];
    const TileCoord tc = tile_coord(A.g, (int64_t)blockIdx.x - B.tile_start[mi]);
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
            k = k < B.K ? k : B.K - 1;
            p = B.grid.p[k];
        }
        uint8_t* dst = reinterpret_cast<uint8_t*>(wrow);   // packed in place, behind the read position
        const uint8_t* __restrict__ mrow =
            A.mask != nullptr ? A.mask + (tc.row0 + lane) * A.mask_ld + (tc.col0 >> 3) : nullptr;
        float sc = 0.0f, of = 0.0f;
        switch (a) {
            case 1: quantize_uniform<DT, 8>(wrow, mrow, G, p, dst, &sc, &of); break;
            case 2: quantize_uniform<DT, 4>(wrow, mrow, G, p, dst, &sc, &of); break;
            case 3: quantize_uniform<DT, 3>(wrow, mrow, G, p, dst, &sc, &of); break;
            case 4: quantize_uniform<DT, 2>(wrow, mrow, G, p, dst, &sc, &of); break;
            case 5: quantize_ternary<DT>(wrow, mrow, G, dst, &sc); break;
            default: quantize_binary<DT>(wrow, mrow, G, dst, &sc); break;
        }
        A.scale[gidx] = sc;
        A.offset[gidx] = of;
    }
    __syncthreads();

    copy_out_rows(tile, row_bytes, (int32_t)bpg, tc.nrows, A.codes + base + tc.lrow0 * bpg, lane, AP_THREADS);
    // zero the padding that rounds the unit's payload up to 16 bytes
    if (padded != payload && tc.t == A.g.tiles_per_unit - 1 && lane < padded - payload)
        A.codes[base + payload + lane] = 0;
}

// ---------------------------------------------------------------------------------------
// Fast path: bf16, chunk_w = 8 * LPR with LPR = 4, 8 or 16 (chunk 32, 64, 128).  LPR
// adjacent lanes share one row: a lane loads 16 bytes (8 weights) straight into registers
// -- a wave instruction covers 64 / LPR rows with fully coalesced segments -- and the
// row's min / max / sum |w| are combined across its lanes with DPP butterflies.  A wave
// owns 16 rows of the 64-row tile and issues all of its loads before the first use, so the
// arithmetic of one piece overlaps the arrival of the next and of the other waves' pieces;
// with ~40 VGPRs and at most 8 KB of LDS, 32 waves fit on a CU.  Each lane packs its own
// eight codes (8, 4, 2 or 1 bytes: one store; 3-bit codes: three lanes of a quad store one
// dword each) and stores them to consecutive addresses.  Only the base-3 bytes, which
// straddle lane boundaries, are regrouped through LDS.  The per-row divisions are taken
// once per wave: lane `piece` of a row derives the parameters of the row's piece-th
// iteration and the others fetch them with a quad broadcast.
//
// The sum of |w| is combined in a tree here, not in column order.  Both orders give the
// exact sum, hence the same fp64 value, while every partial sum is representable: all
// |w| are multiples of 2^(Emin-134) and the sum is below 2^(Emax-126) * chunk_w, so
// Emax - Emin <= 36 suffices.  A row that fails the test is summed again in column order.
constexpr int APS_THREADS = 256;
constexpr int APS_WAVE_ROWS = 16;

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x) {
    // (every lane has a source lane under the controls used here; bound_ctrl only tells the
    // compiler that the destination needs no initial value)
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
    return __uint_as_float(dpp_u32<CTRL>(__float_as_uint(x)));
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x) {
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    const uint64_t r = (uint64_t)dpp_u32<CTRL>((uint32_t)b) | ((uint64_t)dpp_u32<CTRL>((uint32_t)(b >> 32)) << 32);
    return __longlong_as_double((long long)r);
}
constexpr int DPP_XOR1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141;  // lane i <- lane 7 - i of each 8
constexpr int DPP_MIRROR = 0x140;       // lane i <- lane 15 - i of each 16
constexpr int DPP_QUAD_NEXT = 0xF9;     // quad_perm [1,2,3,3]

// All-reduce over the LPR lanes of a row (LPR-aligned lane groups inside a 16-lane DPP row).
#define WINDQ_ROW_REDUCE(NAME, T, DPPFN, COMBINE)                              \
    template <int LPR>                                                         \
    __device__ __forceinline__ T NAME(T x) {                                   \
        { const T y = DPPFN<DPP_XOR1>(x); x = COMBINE; }                       \
        { const T y = DPPFN<DPP_XOR2>(x); x = COMBINE; }                       \
        if (LPR >= 8) { const T y = DPPFN<DPP_HALF_MIRROR>(x); x = COMBINE; }  \
        if (LPR >= 16) { const T y = DPPFN<DPP_MIRROR>(x); x = COMBINE; }      \
        return x;                                                              \
    }
WINDQ_ROW_REDUCE(row_min_f32, float, dpp_f32, fminf(x, y))
WINDQ_ROW_REDUCE(row_max_f32, float, dpp_f32, fmaxf(x, y))
WINDQ_ROW_REDUCE(row_min_u32, uint32_t, dpp_u32, (x < y ? x : y))
WINDQ_ROW_REDUCE(row_max_u32, uint32_t, dpp_u32, (x > y ? x : y))
WINDQ_ROW_REDUCE(row_sum_f64, double, dpp_f64, x + y)
WINDQ_ROW_REDUCE(row_sum_u32, uint32_t, dpp_u32, x + y)
#undef WINDQ_ROW_REDUCE

constexpr int DPP_ROR4 = 0x124;         // lane i <- lane (i + 4) mod 16 of its row of 16
constexpr int DPP_ROR8 = 0x128;
template <int CTRL> __device__ __forceinline__ uint32_t dpp_any(uint32_t x) { return dpp_u32<CTRL>(x); }
template <int CTRL> __device__ __forceinline__ float dpp_any(float x) { return dpp_f32<CTRL>(x); }
template <int CTRL> __device__ __forceinline__ double dpp_any(double x) { return dpp_f64<CTRL>(x); }

// Sixteen lanes share a row and hold four values each (one per iteration): reduces value k over
// the sixteen lanes and leaves the result in the lanes with (piece & 3) == k, the ones that
// derive the parameters of iteration k.  Lanes trade the values they do not keep (two, then one)
// inside their quad, then the four quads combine by rotation: 5 combining steps per lane where
// four all-reduces take 16.  The order of combination differs from a butterfly's; it is used
// only for exact sums and for min / max.
template <typename T, typename Op>
__device__ __forceinline__ T row_scatter_reduce16(const T (&v)[4], int piece, Op op) {
    const bool b0 = (piece & 1) != 0, b1 = (piece & 2) != 0;
    T keep_a = b0 ? v[1] : v[0], send_a = b0 ? v[0] : v[1];
    T keep_b = b0 ? v[3] : v[2], send_b = b0 ? v[2] : v[3];
    keep_a = op(keep_a, dpp_any<DPP_XOR1>(send_a));
    keep_b = op(keep_b, dpp_any<DPP_XOR1>(send_b));
    T keep = b1 ? keep_b : keep_a;
    const T send = b1 ? keep_a : keep_b;
    keep = op(keep, dpp_any<DPP_XOR2>(send));
    keep = op(keep, dpp_any<DPP_ROR8>(keep));
    keep = op(keep, dpp_any<DPP_ROR4>(keep));
    return keep;
}

// Value held by lane IT of the caller's quad.
template <int IT>
__device__ __forceinline__ float quad_bcast(float x) {
    return dpp_f32<IT * 0x55>(x);
}

__device__ __forceinline__ void unpack8(const uint4& raw, float (&w)[8]) {
    w[0] = bf16_bits_to_f32(raw.x & 0xffffu); w[1] = __uint_as_float(raw.x & 0xffff0000u);
    w[2] = bf16_bits_to_f32(raw.y & 0xffffu); w[3] = __uint_as_float(raw.y & 0xffff0000u);
    w[4] = bf16_bits_to_f32(raw.z & 0xffffu); w[5] = __uint_as_float(raw.z & 0xffff0000u);
    w[6] = bf16_bits_to_f32(raw.w & 0xffffu); w[7] = __uint_as_float(raw.w & 0xffff0000u);
}

// Byte `sel` of `old` replaced by the integer value of f (f is an exact integer in [0, 255]).
__device__ __forceinline__ uint32_t put_byte(float f, uint32_t sel, uint32_t old) {
    return __builtin_amdgcn_cvt_pk_u8_f32(f, sel, old);
}

// Where one lane sits in its workgroup's tile.
template <int LPR>
struct SplitLane {
    static constexpr int RPI = 64 / LPR;             // rows per wave instruction
    static constexpr int NI = APS_WAVE_ROWS / RPI;   // instructions (iterations) per wave: 1, 2 or 4
    int piece;                                       // which 8 columns of the row
    int row0;                                        // tile row of iteration 0; iteration it adds it * RPI
    int sel;                                         // the iteration whose row parameters this lane derives
    __device__ __forceinline__ explicit SplitLane(int tid) {
        const int lane = tid & 63;
        piece = lane % LPR;
        row0 = (tid >> 6) * APS_WAVE_ROWS + lane / LPR;
        sel = piece & (NI - 1);
    }
};

// `prot` (here and below): per iteration, the protection bits of the lane's eight columns
// (one byte of the mask; 0 everywhere when MASKED is false).
template <int LPR, int BITS, bool MASKED>
__device__ __forceinline__ void split_uniform(const ApplyArgs& A, const TileCoord& tc, const SplitLane<LPR>& L,
                                              const uint4 (&raw)[SplitLane<LPR>::NI],
                                              const uint32_t (&prot)[SplitLane<LPR>::NI], float p,
                                              uint8_t* __restrict__ out, int64_t bpg) {
    constexpr int NI = SplitLane<LPR>::NI, RPI = SplitLane<LPR>::RPI;
    float w[8];
    float smn = 0.0f, smx = 0.0f;
    float mns[NI], mxs[NI];
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        unpack8(raw[it], w);
        float mn, mx;
        if (!MASKED) {
            mn = fminf(fminf(fminf(w[0], w[1]), fminf(w[2], w[3])), fminf(fminf(w[4], w[5]), fminf(w[6], w[7])));
            mx = fmaxf(fmaxf(fmaxf(w[0], w[1]), fmaxf(w[2], w[3])), fmaxf(fmaxf(w[4], w[5]), fmaxf(w[6], w[7])));
        } else {
            mn = INFINITY;
            mx = -INFINITY;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool kept = ((prot[it] >> j) & 1u) == 0u;
                mn = fminf(mn, kept ? w[j] : INFINITY);
                mx = fmaxf(mx, kept ? w[j] : -INFINITY);
            }
        }
        mns[it] = mn;
        mxs[it] = mx;
    }
    if constexpr (NI == 4) {
        smn = row_scatter_reduce16(mns, L.piece, [](float x, float y) { return fminf(x, y); });
        smx = row_scatter_reduce16(mxs, L.piece, [](float x, float y) { return fmaxf(x, y); });
    } else {
#pragma unroll
        for (int it = 0; it < NI; ++it) {
            const float mn = row_min_f32<LPR>(mns[it]);
            const float mx = row_max_f32<LPR>(mxs[it]);
            if (it == 0 || L.sel == it) {
                smn = mn;
                smx = mx;
            }
        }
    }
    if (MASKED && smn > smx) smn = smx = 0.0f;      // no weight of the group is kept
    const float qmax = (float)((1 << BITS) - 1);
    const float lo = p * smn;
    const float hi = p * smx;
    const float rg = hi - lo;
    float d = rg / qmax;
    const bool ok = d >= FLT_MIN;
    d = ok ? d : 0.0f;
    const float inv = ok ? 1.0f / d : 0.0f;
    if (L.piece < NI) {
        const int r = L.row0 + L.piece * RPI;
        if (r < tc.nrows) {
            const int64_t gidx = tc.u * A.g.R_u + tc.lrow0 + r;
            A.scale[gidx] = d;
            A.offset[gidx] = lo;
        }
    }
    auto one = [&](auto IT) {
        constexpr int it = decltype(IT)::value;
        const float lo_r = NI == 1 ? lo : quad_bcast<it>(lo);
        const float inv_r = NI == 1 ? inv : quad_bcast<it>(inv);
        unpack8(raw[it], w);
        float q[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float u = w[j] - lo_r;
            const float t = u * inv_r;
            q[j] = __builtin_amdgcn_fmed3f(__builtin_rintf(t), 0.0f, qmax);
            if (MASKED && ((prot[it] >> j) & 1u) != 0u) q[j] = 0.0f;      // placeholder in a protected slot
        }
        const int r = L.row0 + it * RPI;
        const bool valid = r < tc.nrows;
        uint8_t* dst = out + r * bpg;
        if constexpr (BITS == 8) {
            const uint32_t v0 = put_byte(q[0], 0, put_byte(q[1], 1, put_byte(q[2], 2, put_byte(q[3], 3, 0u))));
            const uint32_t v1 = put_byte(q[4], 0, put_byte(q[5], 1, put_byte(q[6], 2, put_byte(q[7], 3, 0u))));
            if (valid) *reinterpret_cast<uint2*>(dst + L.piece * 8) = make_uint2(v0, v1);
        } else if constexpr (BITS == 4) {
            const float b0 = fmaf(q[1], 16.0f, q[0]), b1 = fmaf(q[3], 16.0f, q[2]);
            const float b2 = fmaf(q[5], 16.0f, q[4]), b3 = fmaf(q[7], 16.0f, q[6]);
            const uint32_t v = put_byte(b0, 0, put_byte(b1, 1, put_byte(b2, 2, put_byte(b3, 3, 0u))));
            if (valid) *reinterpret_cast<uint32_t*>(dst + L.piece * 4) = v;
        } else if constexpr (BITS == 2) {
            float v = q[7];
#pragma unroll
            for (int j = 6; j >= 0; --j) v = fmaf(v, 4.0f, q[j]);
            if (valid) *reinterpret_cast<uint16_t*>(dst + L.piece * 2) = (uint16_t)(uint32_t)v;
        } else {   // 3 bits: eight codes = 24 bits, exact in fp32; a quad's 12 bytes leave as 3 dwords
            float v = q[7];
#pragma unroll
            for (int j = 6; j >= 0; --j) v = fmaf(v, 8.0f, q[j]);
            const uint32_t mine = (uint32_t)v;
            const uint32_t next = dpp_u32<DPP_QUAD_NEXT>(mine);
            const int j = L.piece & 3;
            const uint32_t dw = j == 0 ? (mine | (next << 24)) : (j == 1 ? ((mine >> 8) | (next << 16)) : ((mine >> 16) | (next << 8)));
            if (valid && j < 3) *reinterpret_cast<uint32_t*>(dst + (L.piece >> 2) * 12 + j * 4) = dw;
        }
    };
    one(std::integral_constant<int, 0>{});
    if constexpr (NI >= 2) one(std::integral_constant<int, 1>{});
    if constexpr (NI >= 4) {
        one(std::integral_constant<int, 2>{});
        one(std::integral_constant<int, 3>{});
    }
}

// Mean |w| over the kept weights of the row this lane derives parameters for (iteration
// L.sel), as stored: the fp64 sum divided by the number kept, rounded to fp32; 0 when none is kept.
template <int LPR, bool MASKED>
__device__ __forceinline__ float split_abs_mean(const ApplyArgs& A, const TileCoord& tc, const SplitLane<LPR>& L,
                                                const uint4 (&raw)[SplitLane<LPR>::NI],
                                                const uint32_t (&prot)[SplitLane<LPR>::NI]) {
    constexpr int NI = SplitLane<LPR>::NI, RPI = SplitLane<LPR>::RPI, G = 8 * LPR;
    double sums[NI];
    uint32_t kmaxs[NI], kmins[NI], kepts[NI];
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        float w[8];
        unpack8(raw[it], w);
        double S1 = 0.0;
#pragma unroll
        for (int j = 0; j < 8; ++j) S1 += MASKED && ((prot[it] >> j) & 1u) != 0u ? 0.0 : (double)fabsf(w[j]);
        sums[it] = S1;
        kepts[it] = 8u - (uint32_t)__builtin_popcount(prot[it]);
        // largest magnitude key, and smallest non-zero one less 1 (a zero wraps to 2^32 - 1)
        uint32_t kmax = 0u, kmin = 0xffffffffu;
        const uint32_t dws[4] = {raw[it].x, raw[it].y, raw[it].z, raw[it].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t h = (dws[i] >> 16) & 0x7fffu, l = dws[i] & 0x7fffu;
            kmax = max(kmax, max(h, l));
            kmin = min(kmin, min(h - 1u, l - 1u));
        }
        kmaxs[it] = kmax;
        kmins[it] = kmin;
    }
    // the row of iteration L.sel: its sum, its kept count, its largest and smallest keys
    double S1 = 0.0;
    uint32_t n_kept = G, kmax = 0u, kmin = 0xffffffffu;
    if constexpr (NI == 4) {
        S1 = row_scatter_reduce16(sums, L.piece, [](double x, double y) { return x + y; });
        kmax = row_scatter_reduce16(kmaxs, L.piece, [](uint32_t x, uint32_t y) { return x > y ? x : y; });
        kmin = row_scatter_reduce16(kmins, L.piece, [](uint32_t x, uint32_t y) { return x < y ? x : y; });
        if (MASKED) n_kept = row_scatter_reduce16(kepts, L.piece, [](uint32_t x, uint32_t y) { return x + y; });
    } else {
#pragma unroll
        for (int it = 0; it < NI; ++it) {
            const double s = row_sum_f64<LPR>(sums[it]);
            const uint32_t kx = row_max_u32<LPR>(kmaxs[it]), kn = row_min_u32<LPR>(kmins[it]);
            const uint32_t nk = MASKED ? row_sum_u32<LPR>(kepts[it]) : (uint32_t)G;
            if (it == 0 || L.sel == it) {
                S1 = s;
                kmax = kx;
                kmin = kn;
                n_kept = nk;
            }
        }
    }
    const int emax = (int)(kmax >> 7);
    const int emin = max((int)((kmin + 1u) >> 7), 1);      // (an all-zero row: kmin + 1 wraps to 0, and kmax is 0)
    if (kmax != 0u && emax - emin > 36) {
        // partial sums may round: take the sum in column order instead
        const int r = L.row0 + L.sel * RPI;
        S1 = 0.0;
        if (r < tc.nrows) {
            const uint16_t* __restrict__ wrow =
                static_cast<const uint16_t*>(A.W) + (tc.row0 + r) * A.g.ld + tc.col0;
            const uint8_t* __restrict__ mrow = MASKED ? A.mask + (tc.row0 + r) * A.mask_ld + (tc.col0 >> 3) : nullptr;
            for (int c = 0; c < G; ++c) {
                const bool kept = !MASKED || ((mrow[c >> 3] >> (c & 7)) & 1u) == 0u;
                S1 += kept ? (double)fabsf(bf16_bits_to_f32(wrow[c])) : 0.0;
            }
        }
    }
    return n_kept > 0u ? (float)(S1 / (double)n_kept) : 0.0f;
}

template <int LPR, bool MASKED>
__device__ __forceinline__ void split_ternary(const ApplyArgs& A, const TileCoord& tc, const SplitLane<LPR>& L,
                                              const uint4 (&raw)[SplitLane<LPR>::NI],
                                              const uint32_t (&prot)[SplitLane<LPR>::NI], uint8_t* __restrict__ out,
                                              uint8_t* trits) {
    constexpr int NI = SplitLane<LPR>::NI, RPI = SplitLane<LPR>::RPI, G = 8 * LPR, NB = (G + 4) / 5;
    float gamma = split_abs_mean<LPR, MASKED>(A, tc, L, raw, prot);
    const bool ok = gamma >= FLT_MIN;
    gamma = ok ? gamma : 0.0f;
    const float inv = ok ? 1.0f / gamma : 0.0f;
    if (L.piece < NI) {
        const int r = L.row0 + L.piece * RPI;
        if (r < tc.nrows) {
            const int64_t gidx = tc.u * A.g.R_u + tc.lrow0 + r;
            A.scale[gidx] = gamma;
            A.offset[gidx] = 0.0f;
        }
    }
    // trits (q + 1) as bytes, rows of G bytes: lane l of iteration it writes bytes [8 * (64 * it + l), +8)
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint8_t* wt = trits + wave * (APS_WAVE_ROWS * G);
    auto one = [&](auto IT) {
        constexpr int it = decltype(IT)::value;
        const float inv_r = NI == 1 ? inv : quad_bcast<it>(inv);
        float w[8];
        unpack8(raw[it], w);
        float q[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float t = w[j] * inv_r;
            q[j] = __builtin_amdgcn_fmed3f(__builtin_rintf(t), -1.0f, 1.0f) + 1.0f;
            if (MASKED && ((prot[it] >> j) & 1u) != 0u) q[j] = 0.0f;      // placeholder in a protected slot
        }
        const uint32_t v0 = put_byte(q[0], 0, put_byte(q[1], 1, put_byte(q[2], 2, put_byte(q[3], 3, 0u))));
        const uint32_t v1 = put_byte(q[4], 0, put_byte(q[5], 1, put_byte(q[6], 2, put_byte(q[7], 3, 0u))));
        *reinterpret_cast<uint2*>(wt + 8 * (64 * it + lane)) = make_uint2(v0, v1);
    };
    one(std::integral_constant<int, 0>{});
    if constexpr (NI >= 2) one(std::integral_constant<int, 1>{});
    if constexpr (NI >= 4) {
        one(std::integral_constant<int, 2>{});
        one(std::integral_constant<int, 3>{});
    }
    __syncthreads();
    // five trits -> one byte; the wave's 16 rows x NB bytes are consecutive in the code stream
    // and start on a multiple of 16 * NB bytes, so they leave as whole dwords (16 * NB is a
    // multiple of 4); in a ragged last tile the bytes of the rows past the end are not written.
    const int wrow0 = wave * APS_WAVE_ROWS;
    const int n_valid = tc.nrows - wrow0 < 0 ? 0 : (tc.nrows - wrow0 < APS_WAVE_ROWS ? tc.nrows - wrow0 : APS_WAVE_ROWS);
    const int valid_bytes = n_valid * NB;
    uint8_t* __restrict__ wout = out + (int64_t)wrow0 * NB;
    for (int d = lane; d < APS_WAVE_ROWS * NB / 4; d += 64) {
        uint32_t word = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int b = 4 * d + k;
            const int r = b / NB, j = b - r * NB;
            const uint8_t* t5 = wt + r * G + 5 * j;
            uint32_t v = t5[0];
            if (5 * j + 1 < G) v += 3u * t5[1];
            if (5 * j + 2 < G) v += 9u * t5[2];
            if (5 * j + 3 < G) v += 27u * t5[3];
            if (5 * j + 4 < G) v += 81u * t5[4];
            word |= v << (8 * k);
        }
        if (4 * d + 4 <= valid_bytes) {
            *reinterpret_cast<uint32_t*>(wout + 4 * d) = word;
        } else {
            for (int k = 0; k < 4; ++k)
                if (4 * d + k < valid_bytes) wout[4 * d + k] = (uint8_t)(word >> (8 * k));
        }
    }
}

template <int LPR, bool MASKED>
__device__ __forceinline__ void split_binary(const ApplyArgs& A, const TileCoord& tc, const SplitLane<LPR>& L,
                                             const uint4 (&raw)[SplitLane<LPR>::NI],
                                             const uint32_t (&prot)[SplitLane<LPR>::NI], uint8_t* __restrict__ out) {
    constexpr int NI = SplitLane<LPR>::NI, RPI = SplitLane<LPR>::RPI;
    const float alpha = split_abs_mean<LPR, MASKED>(A, tc, L, raw, prot);
    if (L.piece < NI) {
        const int r = L.row0 + L.piece * RPI;
        if (r < tc.nrows) {
            const int64_t gidx = tc.u * A.g.R_u + tc.lrow0 + r;
            A.scale[gidx] = alpha;
            A.offset[gidx] = 0.0f;
        }
    }
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        float w[8];
        unpack8(raw[it], w);
        uint32_t byte = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) byte |= (w[j] >= 0.0f ? 1u : 0u) << j;
        const int r = L.row0 + it * RPI;
        if (r < tc.nrows) out[r * LPR + L.piece] = (uint8_t)(byte & ~prot[it]);
    }
}

// tile_coord in 32-bit arithmetic (the host keeps n_tiles below 2^31).
__device__ __forceinline__ TileCoord tile_coord32(const Geometry& g, uint32_t tile) {
    const uint32_t n_chunks = (uint32_t)g.n_chunks, tpu = (uint32_t)g.tiles_per_unit;
    TileCoord tc;
    const uint32_t band = tile / n_chunks, j = tile - band * n_chunks;
    const uint32_t rb = band / tpu, t = band - rb * tpu;
    tc.t = t;
    tc.u = (int64_t)rb * n_chunks + j;
    tc.lrow0 = (int64_t)t * TILE_ROWS;
    tc.row0 = rb * g.R_u + tc.lrow0;
    const int64_t left = g.R_u - tc.lrow0;
    tc.nrows = left < TILE_ROWS ? (int32_t)left : TILE_ROWS;
    tc.col0 = (int64_t)j * g.chunk_w;
    return tc;
}

template <int LPR, bool MASKED>
__global__ __launch_bounds__(APS_THREADS, MASKED ? 6 : 7) void apply_plan_split_kernel(const ApplyBatch B) {
    constexpr int G = 8 * LPR, NI = SplitLane<LPR>::NI, RPI = SplitLane<LPR>::RPI;
    __shared__ __attribute__((aligned(16))) uint8_t trits[TILE_ROWS * G];
    const int mi = batch_index(B.tile_start, B.n, blockIdx.x);
    const ApplyArgs& A = B.m[mi];
    const TileCoord tc = tile_coord32(A.g, (uint32_t)((int64_t)blockIdx.x - B.tile_start[mi]));
    const SplitLane<LPR> L(threadIdx.x);

    int a = A.action[tc.u];
    if (a >= WINDQ_N_ACTIONS) a = 0;
    const int64_t bpg = dev_bytes_per_group(a, G);
    const int64_t base = A.code_off[tc.u];
    const int64_t payload = bpg * A.g.R_u;
    const int64_t padded = (payload + 15) & ~(int64_t)15;
    if (base < 0 || (base & 15) != 0 || base + padded > A.codes_bytes) a = 0;
    if (a == 0) {
        if (threadIdx.x < tc.nrows) {
            const int64_t gidx = tc.u * A.g.R_u + tc.lrow0 + threadIdx.x;
            A.scale[gidx] = 0.0f;
            A.offset[gidx] = 0.0f;
        }
        return;
    }

    uint4 raw[NI];
    uint32_t prot[NI];
    const char* __restrict__ wbase = static_cast<const char*>(A.W);
#pragma unroll
    for (int it = 0; it < NI; ++it) {
        const int r = L.row0 + it * RPI;
        raw[it] = make_uint4(0u, 0u, 0u, 0u);
        prot[it] = 0u;
        if (r < tc.nrows) {
            raw[it] = *reinterpret_cast<const uint4*>(wbase + ((tc.row0 + r) * A.g.ld + tc.col0) * 2 + L.piece * 16);
            if (MASKED) prot[it] = A.mask[(tc.row0 + r) * A.mask_ld + (tc.col0 >> 3) + L.piece];
        }
    }

    float p = 1.0f;
    if (a <= 4 && A.clip_idx != nullptr) {
        int k = A.clip_idx[tc.u * 4 + (a - 1)];
        k = k < B.K ? k : B.K - 1;
        p = B.grid.p[k];
    }
    uint8_t* __restrict__ out = A.codes + base + tc.lrow0 * bpg;   // the tile's rows, bpg bytes each
    switch (a) {
        case 1: split_uniform<LPR, 8, MASKED>(A, tc, L, raw, prot, p, out, bpg); break;
        case 2: split_uniform<LPR, 4, MASKED>(A, tc, L, raw, prot, p, out, bpg); break;
        case 3: split_uniform<LPR, 3, MASKED>(A, tc, L, raw, prot, p, out, bpg); break;
        case 4: split_uniform<LPR, 2, MASKED>(A, tc, L, raw, prot, p, out, bpg); break;
        case 5: split_ternary<LPR, MASKED>(A, tc, L, raw, prot, out, trits); break;
        default: split_binary<LPR, MASKED>(A, tc, L, raw, prot, out); break;
    }
    // zero the padding that rounds the unit's payload up to 16 bytes
    if (padded != payload && tc.t == A.g.tiles_per_unit - 1 && (int64_t)threadIdx.x < padded - payload)
        A.codes[base + payload + threadIdx.x] = 0;
}

}  // namespace windq

using namespace windq;

// One matrix of a launch as the entry points see it.
struct ApplyItem {
    const windq_mat* W;
    const uint8_t* mask;
    const uint8_t* action;
    const uint8_t* clip_idx;
    const int64_t* code_off;
    uint8_t* codes;
    size_t codes_bytes;
    float* scale;
    float* offset;
    void* ws;
    size_t ws_bytes;
};

static int apply_plan_launch(const ApplyItem* items, int32_t n, int32_t chunk_w, int64_t unit_rows, const float* clip_grid,
                             int32_t K, void* stream) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    ApplyBatch B;
    B.n = n;
    bool any_idx = false;
    for (int32_t i = 0; i < n; ++i) any_idx = any_idx || items[i].clip_idx != nullptr;
    int st;
    if (any_idx || clip_grid != nullptr) {
        st = check_clip_grid(clip_grid, K);
        if (st != WINDQ_OK) return st;
    } else {
        K = 1;
    }
    B.K = K;
    for (int k = 0; k < WINDQ_MAX_CLIP; ++k) B.grid.p[k] = clip_grid != nullptr ? clip_grid[k < K ? k : K - 1] : 1.0f;
    const bool masked = items[0].mask != nullptr;
    int64_t tiles = 0;
    for (int32_t i = 0; i < n; ++i) {
        const ApplyItem& it = items[i];
        ApplyArgs& A = B.m[i];
        if (it.W == nullptr) return WINDQ_EINVAL;
        st = make_geometry(it.W, chunk_w, unit_rows, &A.g);
        if (st != WINDQ_OK) return st;
        if (it.action == nullptr || it.code_off == nullptr || it.scale == nullptr || it.offset == nullptr) return WINDQ_EINVAL;
        if (it.codes == nullptr && it.codes_bytes != 0) return WINDQ_EINVAL;
        if (it.codes != nullptr && !aligned(it.codes, 16)) return WINDQ_EINVAL;
        if (!aligned(it.code_off, 8)) return WINDQ_EINVAL;
        if (it.W->dtype != items[0].W->dtype || (it.mask != nullptr) != masked) return WINDQ_EINVAL;   // one kernel per launch
        if (it.ws == nullptr || it.ws_bytes < apply_ws_bytes(A.g) || !aligned(it.ws, 256)) return WINDQ_EWORKSPACE;
        A.W = it.W->data;
        A.mask = it.mask;
        A.mask_ld = it.W->cols / 8;
        A.action = it.action;
        A.clip_idx = clip_grid != nullptr ? it.clip_idx : nullptr;
        A.code_off = it.code_off;
        A.codes = it.codes;
        A.codes_bytes = (int64_t)it.codes_bytes;
        A.scale = it.scale;
        A.offset = it.offset;
        B.tile_start[i] = tiles;
        tiles += A.g.n_tiles;
    }
    for (int32_t i = n; i <= WINDQ_MAX_BATCH; ++i) B.tile_start[i] = tiles;
    for (int32_t i = n; i < WINDQ_MAX_BATCH; ++i) B.m[i] = B.m[0];
    if (tiles > (int64_t)0x7fffffff) return WINDQ_ESHAPE;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int32_t dtype = items[0].W->dtype;
    const size_t lds = raw_tile_lds_bytes(dtype, chunk_w);
    const dim3 grid((unsigned)tiles);
    const bool fast = dtype == WINDQ_BF16;
    auto launch_split = [&](auto plain, auto prot) {
        if (masked) hipLaunchKernelGGL(prot, grid, dim3(APS_THREADS), 0, hs, B);
        else hipLaunchKernelGGL(plain, grid, dim3(APS_THREADS), 0, hs, B);
    };
    if (fast && chunk_w == 128) {
        launch_split(&apply_plan_split_kernel<16, false>, &apply_plan_split_kernel<16, true>);
    } else if (fast && chunk_w == 64) {
        launch_split(&apply_plan_split_kernel<8, false>, &apply_plan_split_kernel<8, true>);
    } else if (fast && chunk_w == 32 && !masked) {      // (masked at this width: the general kernel below)
        hipLaunchKernelGGL((apply_plan_split_kernel<4, false>), grid, dim3(APS_THREADS), 0, hs, B);
    } else if (dtype == WINDQ_BF16) {
        st = ensure_lds(reinterpret_cast<const void*>(&apply_plan_kernel<WINDQ_BF16>), lds);
        if (st != WINDQ_OK) return st;
        hipLaunchKernelGGL(apply_plan_kernel<WINDQ_BF16>, grid, dim3(AP_THREADS), lds, hs, B);
    } else {
        st = ensure_lds(reinterpret_cast<const void*>(&apply_plan_kernel<WINDQ_F32>), lds);
        if (st != WINDQ_OK) return st;
        hipLaunchKernelGGL(apply_plan_kernel<WINDQ_F32>, grid, dim3(AP_THREADS), lds, hs, B);
    }
    if (hipPeekAtLastError() != hipSuccess) return WINDQ_EHIP;
    return WINDQ_OK;
}

static int apply_plan_impl(const windq_mat* W, int32_t chunk_w, int64_t unit_rows, const uint8_t* mask,
                           const uint8_t* action, const uint8_t* clip_idx, const float* clip_grid, int32_t K,
                           const int64_t* code_off, uint8_t* codes, size_t codes_bytes, float* scale, float* offset,
                           void* ws, size_t ws_bytes, void* stream) {
    if (W == nullptr) return WINDQ_EINVAL;
    const ApplyItem it = {W, mask, action, clip_idx, code_off, codes, codes_bytes, scale, offset, ws, ws_bytes};
    return apply_plan_launch(&it, 1, chunk_w, unit_rows, clip_grid, K, stream);
}

extern "C" int windq_apply_plan(const windq_mat* W, int32_t chunk_w, int64_t unit_rows, const uint8_t* action,
                                const uint8_t* clip_idx, const float* clip_grid, int32_t K, const int64_t* code_off,
                                uint8_t* codes, size_t codes_bytes, float* scale, float* offset, void* ws,
                                size_t ws_bytes, void* stream) {
    return apply_plan_impl(W, chunk_w, unit_rows, nullptr, action, clip_idx, clip_grid, K, code_off, codes, codes_bytes,
                           scale, offset, ws, ws_bytes, stream);
}

extern "C" int windq_apply_plan_prot(const windq_mat* W, int32_t chunk_w, int64_t unit_rows, const uint8_t* mask,
                                     const uint8_t* action, const uint8_t* clip_idx, const float* clip_grid, int32_t K,
                                     const int64_t* code_off, uint8_t* codes, size_t codes_bytes, float* scale,
                                     float* offset, void* ws, size_t ws_bytes, void* stream) {
    if (mask == nullptr) return WINDQ_EINVAL;
    return apply_plan_impl(W, chunk_w, unit_rows, mask, action, clip_idx, clip_grid, K, code_off, codes, codes_bytes,
                           scale, offset, ws, ws_bytes, stream);
}

extern "C" int windq_apply_plan_batch(const windq_apply_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows,
                                      const float* clip_grid, int32_t K, void* stream) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    ApplyItem its[WINDQ_MAX_BATCH];
    for (int32_t i = 0; i < n; ++i)
        its[i] = {items[i].W, items[i].mask, items[i].action, items[i].clip_idx, items[i].code_off, items[i].codes,
                  items[i].codes_bytes, items[i].scale, items[i].offset, items[i].ws, items[i].ws_bytes};
    return apply_plan_launch(its, n, chunk_w, unit_rows, clip_grid, K, stream);
}
