// windq_fit_score_all_bits: fit the lightweight quantizer of every unit at all six
// bit-widths and score each fit by the activation-aware reconstruction error
// (Sec. 3.5 "Quantization Engine and Bit Accounting"; App. "Per-unit Scale
// Optimization": per-group scales, group size = chunk size).
//
// Work per weight: 4 bit-widths x K clip ratios + ternary + binary = 4K+2 candidate
// quantizers.  At K = 20 that is ~400 vector instructions per 2-byte weight: the kernel
// is bound by the vector ALU, not by HBM, by a factor of ~30.  So the design minimises
// issue cycles per candidate, using what measurement shows about gfx950's vector ALU:
// v_fma/mul/add/sub_f32 whose operands are all plain VGPRs issue about 1.7x faster than
// any other vector instruction (fp64, min/max/med3, rounding, conversions, anything with
// an SGPR, literal or negated operand), provided >= 4-5 wavefronts are resident per SIMD.
// Hence:
//   * lane-per-group (see windq_common.hpp): quantizer parameters are lane-private and
//     live in VGPRs; the wave-uniform s_c is staged in LDS and read back into VGPRs,
//     constants are pinned in VGPRs;
//   * the hot loop is made of fast fp32 FMA/ADD/MUL only:
//       x  = clamp01(w/range + h)               position in the clipped range; one FMA with
//                                               the free [0,1] output clamp
//       u' = s_c*w - s_c*lo                     one FMA per clip ratio
//       per bit-width b:  tM = x * (2^b-1) + 2^23      rounds to the nearest code (RNE)
//                         q' = tM * s_c - 2^23 s_c     = s_c * code, one rounding
//                         r' = q' * (-step_b) + u'     = s_c * (w - lo - code*step_b)
//                         acc_b += r' * r'
//     4 instructions per candidate and no separate clamp of the code (x is already in
//     [0,1]): 18 per (weight, clip ratio) when all four bit-widths go this short way;
//   * at 8 bits the residual is ~1/500 of (w - lo), so the fp32 roundings of s_c*w,
//     s_c*(w - lo) and s_c*code show in it: ~1e-4 of its size per weight, random in sign.
//     An EXACT 8-bit route, 20 instructions, forms the residual unscaled, relative to an
//     anchor c = lo + q0*step, the grid point nearest zero, as (w - (code - q0)*step) - c,
//     where the FMA rounds once at the small magnitude |c + r|, and only then multiplies by
//     s_c.  (Groups whose weights all have one sign have no grid point near zero: their
//     wavefront uses c = lo and an error-free two-sum of (w - c), 23 instructions.)
//     Which weights may take the short route is decided from the data, at three levels:
//       columns  a column that carries much of the chunk's sum of s_c^2 (above tau times
//                the mean) is listed and scored on the exact route, one column at a time;
//                small units, and chunks with many such columns, sweep every column exactly;
//       rows     a tile in which one row holds more than two thirds of the rows' squared
//                ranges takes the exact sweep;
//       units    every tile that used the short route also sums, per clip index, the
//                variance its roundings can have put into the 8-bit error (see
//                NOISE_MAX below); the finalize kernel adds these up per unit and, where
//                the standard deviation exceeds NOISE_MAX of the unit's 8-bit error at the
//                chosen clip index, puts the unit on a list; a second pair of launches
//                scores the 8-bit candidates of the listed units again, exact route only,
//                and finalizes them again.  With nothing listed those launches end at once.
//   * lanes accumulate in fp32 over the chunk's columns only (<= 512 terms); rows are
//     combined in fp64 in a fixed order (LDS transpose), tiles by the finalize kernel;
//   * what depends on s alone (the column list, s_c of the other columns) is prepared once per
//     chunk by a small kernel ahead of the tiles, which copy it into LDS with their load;
//   * the phases around the sweeps wait more than they issue (loads, barriers, cross-lane
//     chains): they run at a raised wave priority, so that a SIMD's other wavefronts, which are
//     in their sweeps, give up only the few issue slots those phases need.
// Rounding decisions here are taken on x*(2^b-1); windq_apply_plan takes them on
// (w-lo)*(1/step) in fp32.  Where they differ the weight sits within ~3e-5 steps of a
// rounding boundary, where both codes give the same squared error to ~1e-4 of itself,
// and such weights are ~1e-4 of all: the effect on a unit's error is below 1e-7.
// Supported dynamic range: |s_c * w| within fp32's normal range after squaring
// (about 1e-18 .. 1e18); smaller products contribute zero.
#include <float.h>

#include <mutex>
#include <type_traits>
#include <utility>
#include <vector>

#include "windq_common.hpp"
#include "windq_feat.hpp"
#include "windq_ws.hpp"

namespace windq {

constexpr int FS_THREADS = 256;
constexpr int FS_WAVES = FS_THREADS / 64;
constexpr int FS_KB = 5;                    // clip ratios evaluated together by one wavefront pass
constexpr int FS_NRED = FS_KB * 5;          // per-lane sums a pass produces: 4 errors + 1 noise term per clip ratio
constexpr int FS_NEXTRA = 6;                // sums a tile produces once: 3 of the unit features, then ternary / binary / reference
constexpr int FS_NROW = FS_NRED + FS_NEXTRA;    // row of a wavefront's scratch for combining rows
// (Under a mask there are no feature sums, and the row is three columns shorter: with the mask bytes the
// workgroup's LDS would otherwise pass the 32 KB that let five workgroups share a CU.)
__host__ __device__ constexpr int fs_nrow(bool masked) { return masked ? FS_NRED + 3 : FS_NROW; }
constexpr float RNE_POS = 8388608.0f;       // 2^23: x + 2^23 rounds x >= 0 to the nearest-even integer
constexpr int FS_PREP_CHUNKS = FS_THREADS / 64;     // chunks a workgroup of the preparing kernel takes, one per wavefront
constexpr int FS_PREP_CLEAR = FS_THREADS * 4;       // counters one of its workgroups clears
constexpr int FS_REDO_GRID = 512; 
// What a pass over a tile does.
constexpr int FS_SCORE = 0;         // every candidate quantizer
constexpr int FS_ONLY8 = 1;         // the 8-bit candidates alone, exact route (listed units)
constexpr int FS_SCORE_FEAT = 2;    // every candidate, and the first pass of the unit features (Table 1)
constexpr int FS_FEAT_ONLY = 3;     // that first pass alone          // workgroups of the launch that scores listed units again

// The short route's rounding noise in a unit's 8-bit error.  On the short route the residual
// r' = s_c (w - lo - code*step) carries three roundings taken at magnitudes of at most
// s_c*range (range = hi - lo of the group): an error e of variance <= (2^-24 s_c range)^2, of
// random sign.  It moves the squared residual by 2 r' e, so the unit's error moves by a sum
// of variance <= 4 * 2^-48 * sum_rows range^2 * sum_cols s_c^2 r'^2.  Taking r' independent
// of the column (true of rounding residuals), sum_c s_c^2 r'^2 = (S4/S2) * sum_c r'^2 with
// S4 = sum s_c^4, S2 = sum s_c^2 over the columns on the short route; sum_c r'^2 is the lane's
// own 8-bit accumulator.  So every short-route tile emits, per clip index,
//     V = (S4/S2) * sum_rows range^2 * acc8_row,
// and the unit's noise has a standard deviation of at most 2^-23 sqrt(sum_tiles V).  The unit's
// 8-bit candidates are scored again on the exact route when that exceeds NOISE_MAX times the
// unit's 8-bit error at the chosen clip index.  (Measured against fp64, the actual deviation
// is ~0.4 of this estimate: NOISE_MAX = 3e-6 keeps one standard deviation near 1e-6.)
constexpr double NOISE_MAX = 3e-6;
constexpr double NOISE_C1 = 4.0 * 3.552713678800501e-15 / (NOISE_MAX * NOISE_MAX);   // 4 * 2^-48 / NOISE_MAX^2
// A tile takes the exact sweep when one row holds more than 1 / ROW_SHARE of the sum of the
// rows' squared ranges (that row would carry most of the tile's 8-bit error by itself).
constexpr float ROW_SHARE = 1.5f;
constexpr int64_t FS_FEW_ROWS = 64;         // units of fewer rows: the exact sweeps take the normative 8-bit decision

// One matrix of a launch.
struct FitScoreMat {
    const void* W;
    const float* s;
    const uint8_t* mask;   // protection mask [rows][cols/8] (masked kernels only)
    int64_t mask_ld;
    double* partial;       // [n_tiles][5K+12]
    uint32_t* redo_count;  // number of units listed for the exact 8-bit pass
    uint32_t* redo_list;   // [U] their indices, in no particular order
    float* err;            // outputs of the finalize kernel
    uint8_t* clip_idx;
    float* ref_energy;
    Geometry g;
    float tau;         // columns with s_c^2 > tau * mean(s^2) of the chunk take the exact 8-bit route; 0: all do
    float* colsel;     // [n_chunks][colsel_words]: the chunks' column selection, written by the preparing kernel
    // first pass of the unit features (FS_SCORE_FEAT, FS_FEAT_ONLY), else unused
    double* fmoments;      // [n_tiles][4 column quarters][4]: sum w, sum w^2, sum |w|, count(|w| < 1e-6)
    uint32_t* fhist;       // [U][FEAT_BINS]: histogram of the first radix digit of |w|
    uint32_t* ffine;       // bf16: [n_tiles][FEAT_WIN][8] full-resolution counts of the bins around each tile's bulk
    uint32_t* fanchor;     // bf16: [n_tiles] last bin of that record, and (<< 16) the bin of the tile's largest key
    float sparse_thr;      // smallest fp32 that is >= 1e-6
    uint32_t sparse_key;   // bf16: smallest key whose value is >= 1e-6
    uint32_t* fclear;      // the features' counters that start a call at zero, [fclear_words] ...
    int64_t fclear_words;
    uint32_t* flist_count; // ... and one more (bf16), or null
};

// A launch covers up to WINDQ_MAX_BATCH matrices of one chunk width and element type: their
// tiles (and, for the finalize kernel, their units) are numbered one matrix after the other,
// so that one grid keeps the chip filled across matrix boundaries.
struct FitScoreArgs {
    int32_t n;                                   // matrices in the launch
    int32_t K;
    int32_t n_kpass;                             // ceil(K / FS_KB)
    double inv_G;                                // 1 / chunk_w
    int64_t tile_start[WINDQ_MAX_BATCH + 1];     // first tile of matrix i in the grid; [n] = grid size
    int64_t unit_start[WINDQ_MAX_BATCH + 1];
    int64_t prep_start[WINDQ_MAX_BATCH + 1];     // first workgroup of matrix i in the preparing kernel's grid
    FitScoreMat m[WINDQ_MAX_BATCH];
    ClipGrid grid;
};

// LDS of a workgroup, in this order: the raw tile; s_c of the chunk's columns; per wavefront a
// 16 x FS_NROW scratch for combining rows; the column quarters' (min, max) per row; s_c with
// the listed columns zeroed, and the list; the quarters' fp64 sums of |w| per row; under a
// mask, the quarters' kept counts (16 bits each) and the tile's mask bytes.  30.0 KB at G = 128
// (bf16), 31.75 KB under a mask: within the 32 KB that let five workgroups share a CU's 160 KB, on
// purpose: the fast fp32 issue rate needs five resident wavefronts per SIMD (a single
// wavefront issues at most one vector instruction per ~5 cycles).
inline size_t fit_score_lds_bytes(int32_t dtype, int32_t chunk_w, bool masked = false) {
    return raw_tile_lds_bytes(dtype, chunk_w) + (size_t)chunk_w * sizeof(float) +
           (size_t)FS_WAVES * 16 * fs_nrow(masked) * sizeof(float) + (size_t)FS_WAVES * TILE_ROWS * 2 * sizeof(float) +
           (size_t)chunk_w * sizeof(float) + (size_t)FS_HMAX * sizeof(int32_t) +
           (size_t)FS_WAVES * TILE_ROWS * sizeof(double) +
           (masked ? (size_t)FS_WAVES * TILE_ROWS * sizeof(uint16_t) + mask_tile_lds_bytes(chunk_w) : 0);
}

// The 8-bit residual is ~1/500 of the range, so it is taken relative to an ANCHOR c: a grid
// point of the 8-bit quantizer, with the code counted from it (qc = code - q0).
//   ANCHORED (zero lies inside [lo, hi], true for every group of real weight matrices): c is
//   the grid point nearest zero, |c| <= step/2.  Then w - qc*step = c + r is small, the FMA
//   that forms it rounds once at that small magnitude, and subtracting c is exact to the
//   same order: r to ~1e-7 relative in two instructions, no compensation needed.
//   Otherwise (a group whose weights all have one sign) c = lo may be large against the
//   step: (w - c) is split into a rounded value and its rounding error by an error-free
//   two-sum, and the residual is the FMA on the rounded part plus the error.
// A wavefront takes the second route when any of its 64 groups needs it.
struct KParams {
    float rinv, h;     // 1/range; x = (w - a)*rinv + h is the position in the range, a = 0 (anchored) or c.
                       // The sweeps that take every column on the exact route put 1/step of the 8-bit grid
                       // (an IEEE quotient) into h instead, and take x = clamp01((w - lo)*rinv).
    float nc, Mq;      // -c (anchor), 2^23 + q0
    float nlo;         // -lo
    float nd[4];       // -step for 8, 4, 3, 2 bits (0 when degenerate)
};

// The 8-bit code of one weight, less the anchor's code q0, by the normative fp32 steps (the ones
// windq_apply_plan takes): un = fl(w - lo), t = fl(un * fl(1/step)), ties to even, clamped to
// [0, 255].  inv = 1/step; t + 2^23 rounds t >= 0 to the nearest-even integer, and whatever a
// negative t turns into is clamped to code 0.
__device__ __forceinline__ float normative_code8(const float un, const float inv, const float M, const float Mq) {
    const float t = un * inv;         // (two roundings, as the normative steps have them: never one fused operation)
    const float tM = t + M;
    return __builtin_amdgcn_fmed3f(tM, M, M + 255.0f) - Mq;
}

// The exact 8-bit residual of one weight at clip ratio P, times s_c.  NORMATIVE: the code is the
// one the normative steps give (P.h holds 1/step); otherwise it is rne(255 x), which differs from
// it only for a weight within ~2e-5 steps of a tie, where the two residuals have the same
// magnitude to 4e-5: that shows in a unit's error only if a single weight carries a fair share of
// it, so the sweeps over every column, which are the ones small units take, are normative.
template <bool ANCHORED, bool NORMATIVE>
__device__ __forceinline__ float exact_residual8(const float w, const float sc, const KParams& P, const float Q0,
                                                 const float M, float& x) {
    const float base = ANCHORED ? w : w + P.nc;               // w, or w - c rounded
    float fix = P.nc;
    if (!ANCHORED) {
        const float bb = base - w;
        fix = (w - (base - bb)) + (P.nc - bb);                // the rounding error of w - c: (w - c) = base + fix exactly
    }
    float qc;                                                 // code - q0
    if (NORMATIVE) {
        const float un = w + P.nlo;
        x = mul_clamp01(un, P.rinv);                          // position in the clipped range, in [0, 1]
        qc = normative_code8(un, P.h, M, P.Mq);
    } else {
        x = fma_clamp01(base, P.rinv, P.h);
        qc = fmaf(x, Q0, M) - P.Mq;
    }
    return (fmaf(qc, P.nd[0], base) + fix) * sc;              // ((c + r) - c) s_c
}

// One weight against FS_KB clip ratios x 4 bit-widths, the 8-bit one on the exact route.
// sc = s_c, nM = -2^23 (in a VGPR).  Candidate after candidate: the fewest registers, for the sweeps
// that need every parameter of KParams live (all columns on the exact route).
template <bool ANCHORED>
__device__ __forceinline__ void score_weight(const float w, const float sc, const KParams (&P)[FS_KB],
                                             const float (&Q)[4], const float M, const float nM,
                                             float (&acc)[FS_KB][4]) {
    const float w1 = w * sc;
    const float ms = sc * nM;                              // -2^23 * s_c, exact
#pragma unroll
    for (int i = 0; i < FS_KB; ++i) {
        const float u1 = fmaf(P[i].nlo, sc, w1);                  // s_c * (w - lo)
        float x;
        const float r8 = exact_residual8<ANCHORED, false>(w, sc, P[i], Q[0], M, x);
        acc[i][0] = fmaf(r8, r8, acc[i][0]);
#pragma unroll
        for (int b = 1; b < 4; ++b) {
            const float tM = fmaf(x, Q[b], M);
            const float q1 = fmaf(tM, sc, ms);
            const float r1 = fmaf(q1, P[i].nd[b], u1);
            acc[i][b] = fmaf(r1, r1, acc[i][b]);
        }
    }
}

// score_weight with the four bit-widths side by side, stage by stage (see score_weight_short): six live
// temporaries instead of two, for the sweeps over all columns, which read four columns at a time to
// make room for them.  The 8-bit candidate's two extra steps run into the next ratio's first ones.
template <bool ANCHORED, bool NORMATIVE>
__device__ __forceinline__ void score_weight_staged(const float w, const float sc, const KParams (&P)[FS_KB],
                                                    const float (&Q)[4], const float M, const float nM,
                                                    float (&acc)[FS_KB][4]) {
    const float w1 = w * sc;
    const float ms = sc * nM;
#pragma unroll
    for (int i = 0; i < FS_KB; ++i) {
        if constexpr (NORMATIVE) {
            const float u1 = fmaf(P[i].nlo, sc, w1);                  // s_c * (w - lo)
            const float un = w + P[i].nlo;                            // fl(w - lo): the first of the normative steps
            const float x = mul_clamp01(un, P[i].rinv);               // position in the clipped range, in [0, 1]
            float base = w, fix = P[i].nc;
            if (!ANCHORED) {
                const float u0 = w + P[i].nc;                         // w - c, rounded
                const float bb = u0 - w;
                fix = (w - (u0 - bb)) + (P[i].nc - bb);               // its rounding error: (w - c) = u0 + fix exactly
                base = u0;
            }
            // the 8-bit code by the normative steps (P.h = 1/step; see normative_code8), one step per stage
            float t[4];
            __builtin_amdgcn_sched_barrier(0);
            t[0] = un * P[i].h;
#pragma unroll
            for (int b = 1; b < 4; ++b) t[b] = fmaf(x, Q[b], M);
            __builtin_amdgcn_sched_barrier(0);
            t[0] = t[0] + M;
#pragma unroll
            for (int b = 1; b < 4; ++b) t[b] = fmaf(t[b], sc, ms);
            __builtin_amdgcn_sched_barrier(0);
            t[0] = __builtin_amdgcn_fmed3f(t[0], M, M + 255.0f);
#pragma unroll
            for (int b = 1; b < 4; ++b) t[b] = fmaf(t[b], P[i].nd[b], u1);
            __builtin_amdgcn_sched_barrier(0);
            t[0] = t[0] - P[i].Mq;                                    // code - q0
#pragma unroll
            for (int b = 1; b < 4; ++b) acc[i][b] = fmaf(t[b], t[b], acc[i][b]);
            __builtin_amdgcn_sched_barrier(0);
            t[0] = fmaf(t[0], P[i].nd[0], base);                      // (c + r), small
            t[0] = t[0] + fix;                                        // r
            const float r8 = t[0] * sc;
            acc[i][0] = fmaf(r8, r8, acc[i][0]);
        } else {
            const float u1 = fmaf(P[i].nlo, sc, w1);                  // s_c * (w - lo)
            float x, base = w, fix = P[i].nc;
            if (ANCHORED) {
                x = fma_clamp01(w, P[i].rinv, P[i].h);                // position in the clipped range, in [0, 1]
            } else {
                const float u0 = w + P[i].nc;                         // w - c, rounded
                const float bb = u0 - w;
                fix = (w - (u0 - bb)) + (P[i].nc - bb);               // its rounding error: (w - c) = u0 + fix exactly
                x = fma_clamp01(u0, P[i].rinv, P[i].h);
                base = u0;
            }
            float t[4];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < 4; ++b) t[b] = fmaf(x, Q[b], M);
            __builtin_amdgcn_sched_barrier(0);
            t[0] = t[0] - P[i].Mq;                                    // code - q0
#pragma unroll
            for (int b = 1; b < 4; ++b) t[b] = fmaf(t[b], sc, ms);
            __builtin_amdgcn_sched_barrier(0);
            t[0] = fmaf(t[0], P[i].nd[0], base);                      // (c + r), small
#pragma unroll
            for (int b = 1; b < 4; ++b) t[b] = fmaf(t[b], P[i].nd[b], u1);
            __builtin_amdgcn_sched_barrier(0);
            t[0] = t[0] + fix;                                        // r
#pragma unroll
            for (int b = 1; b < 4; ++b) acc[i][b] = fmaf(t[b], t[b], acc[i][b]);
            __builtin_amdgcn_sched_barrier(0);
            const float r8 = t[0] * sc;
            acc[i][0] = fmaf(r8, r8, acc[i][0]);
        }
    }
}

// The 8-bit candidate alone, exact route (the pass over listed units).
template <bool ANCHORED, bool NORMATIVE>
__device__ __forceinline__ void score_weight_8(const float w, const float sc, const KParams (&P)[FS_KB], const float Q0,
                                               const float M, float (&acc)[FS_KB][4]) {
#pragma unroll
    for (int i = 0; i < FS_KB; ++i) {
        float x;
        const float r8 = exact_residual8<ANCHORED, NORMATIVE>(w, sc, P[i], Q0, M, x);
        acc[i][0] = fmaf(r8, r8, acc[i][0]);
    }
}

// The short route: all four bit-widths like the low ones, 18 instructions per (weight, clip
// ratio).  Its 8-bit residual carries the fp32 roundings of s_c*w, s_c*(w - lo) and s_c*code:
// ~1e-4 of its own size per weight, of random sign (see NOISE_MAX for how that is bounded).
__device__ __forceinline__ void score_weight_short(const float w, const float sc, const KParams (&P)[FS_KB],
                                                   const float (&Q)[4], const float M, const float nM,
                                                   float (&acc)[FS_KB][4]) {
    // Instruction ORDER matters as much as instruction count here: the four bit-widths of a clip ratio
    // advance side by side, stage by stage, so that every instruction's inputs are four instructions
    // old and a wavefront does not wait on its own results.  The barriers pin that order (left alone,
    // the compiler finishes one candidate before it starts the next, to save registers: 6 % slower).
    const float w1 = w * sc;
    const float ms = sc * nM;
#pragma unroll
    for (int i = 0; i < FS_KB; ++i) {
        const float u1 = fmaf(P[i].nlo, sc, w1);                  // s_c * (w - lo)
        const float x = fma_clamp01(w, P[i].rinv, P[i].h);        // position in the clipped range, in [0, 1]
        float t[4];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int b = 0; b < 4; ++b) t[b] = fmaf(x, Q[b], M);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int b = 0; b < 4; ++b) t[b] = fmaf(t[b], sc, ms);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int b = 0; b < 4; ++b) t[b] = fmaf(t[b], P[i].nd[b], u1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[i][b] = fmaf(t[b], t[b], acc[i][b]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// One weight of a lane's row at column c.
template <int DT>
__device__ __forceinline__ float read1(const char* __restrict__ wrow, int32_t c) {
    if (DT == WINDQ_BF16) return bf16_bits_to_f32(*reinterpret_cast<const uint16_t*>(wrow + c * 2));
    return *reinterpret_cast<const float*>(wrow + c * 4);
}

// s, or 0 where bit J of the mask byte m is set: the bit, sign-extended to all ones, selects
// between 0 and s (two instructions; written out because the compiler turns the same logic
// back into a three-instruction test-compare-select per weight, and a branch on top).
template <int J>
__device__ __forceinline__ float drop_if_set(float sv, uint32_t m) {
    uint32_t ones;
    asm("v_bfe_i32 %1, %2, %3, 1\n\tv_bfi_b32 %0, %1, 0, %0" : "+v"(sv), "=&v"(ones) : "v"(m), "n"(J));
    return sv;
}
__device__ __forceinline__ void drop_masked(float (&s8)[8], uint32_t m) {
    s8[0] = drop_if_set<0>(s8[0], m); s8[1] = drop_if_set<1>(s8[1], m);
    s8[2] = drop_if_set<2>(s8[2], m); s8[3] = drop_if_set<3>(s8[3], m);
    s8[4] = drop_if_set<4>(s8[4], m); s8[5] = drop_if_set<5>(s8[5], m);
    s8[6] = drop_if_set<6>(s8[6], m); s8[7] = drop_if_set<7>(s8[7], m);
}

// The lane's index in its wavefront, read anew from the hardware at every call (never kept
// in a register between calls).
__device__ __forceinline__ int fresh_lane() {
    int l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    return l;
}

__device__ __forceinline__ float dpp_f32(float x, int ctrl) {
    switch (ctrl) {   // the control word must be a compile-time constant
        case 0xB1: return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
        case 0x4E: return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
        case 0x141: return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xF, 0xF, false));  // row_half_mirror
        default: return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xF, 0xF, false));     // row_mirror
    }
}

// x + (x of the lane whose index differs in bit 0 / bit 1): after both, every lane of a
// quad (4 adjacent rows) holds the quad's sum.
__device__ __forceinline__ float quad_sum(float x) {
    x += dpp_f32(x, 0xB1);
    x += dpp_f32(x, 0x4E);
    return x;
}

// Sum of x over the 64 lanes, the same bits in every lane: quads, then the two quads of a
// half row, the two halves of a row of 16 (DPP mirrors), then the four rows in order.
__device__ __forceinline__ float wave_sum_f32(float x) {
    x = quad_sum(x);
    x += dpp_f32(x, 0x141);
    x += dpp_f32(x, 0x140);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 48));
    return ((r0 + r1) + r2) + r3;
}

// Sums of s[] and maxima of m[] over the 64 lanes, each by the steps of wave_sum_f32 (the same bits
// for a sum), all of them advancing together: a reduction is a chain of dependent cross-lane
// steps that a wavefront waits out one by one, and several chains side by side wait only once.
template <int NS, int NM>
__device__ __forceinline__ void wave_sums_maxes(float (&s)[NS], float (&m)[NM]) {
#pragma unroll
    for (int st = 0; st < 4; ++st) {
        const int ctrl = st == 0 ? 0xB1 : (st == 1 ? 0x4E : (st == 2 ? 0x141 : 0x140));
#pragma unroll
        for (int i = 0; i < NS; ++i) s[i] += dpp_f32(s[i], ctrl);
#pragma unroll
        for (int j = 0; j < NM; ++j) m[j] = fmaxf(m[j], dpp_f32(m[j], ctrl));
    }
    float rs[NS][4], rm[NM][4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
        for (int i = 0; i < NS; ++i) rs[i][r] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s[i]), 16 * r));
#pragma unroll
        for (int j = 0; j < NM; ++j) rm[j][r] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m[j]), 16 * r));
    }
#pragma unroll
    for (int i = 0; i < NS; ++i) s[i] = ((rs[i][0] + rs[i][1]) + rs[i][2]) + rs[i][3];
#pragma unroll
    for (int j = 0; j < NM; ++j) m[j] = fmaxf(fmaxf(rm[j][0], rm[j][1]), fmaxf(rm[j][2], rm[j][3]));
}

// Sums of per-lane fp32 values over the 64 lanes (rows) of a wavefront, in two steps, so that sums
// that become ready at different times share the second.  rows_deposit: N values, quads in fp32 by
// DPP (two adds), the 16 quad sums into columns col0 .. col0+N-1 of the wavefront's private LDS
// scratch.  rows_collect: lane j < n returns the total of column j, the 16 quad sums in fp64 in row
// order.  Fixed order: bit-reproducible.
template <int NROW, int N>
__device__ __forceinline__ void rows_deposit(const float (&v)[N], float* __restrict__ red, int lane, int col0) {
    float qs[N];
#pragma unroll
    for (int j = 0; j < N; ++j) qs[j] = quad_sum(v[j]);
    if ((lane & 3) == 0) {
#pragma unroll
        for (int j = 0; j < N; ++j) red[(lane >> 2) * NROW + col0 + j] = qs[j];
    }
}
template <int NROW>
__device__ __forceinline__ double rows_collect(const float* __restrict__ red, int lane, int n) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    double tot = 0.0;
    if (lane < n) {
#pragma unroll
        for (int i = 0; i < 16; ++i) tot += (double)red[i * NROW + lane];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    return tot;
}

// One tile in one of the FS_* modes.  FS_ONLY8 leaves every other partial of the tile as it is.
// The feature modes add, in the scan that finds the groups' min / max / sum |w| anyway: per
// wavefront (column quarter) the sums of w and w^2 (fp32 per lane over <= 128 weights, products
// of bf16 are exact; fp64 beyond), the count of |w| < 1e-6, and a histogram of |w| in LDS, in
// the space the row-combining scratch uses later.
//   fp32 inputs: the first radix digit of |w| (bits 20-30 of the pattern: exponent + 3 mantissa
//   bits), 2048 bins of 16 bits, two to a dword; added to the unit's histogram in global memory
//   (integer atomics: order does not matter).
//   bf16 inputs: all 15 magnitude bits, key by key, over 198 first-digit bins (2^-21 <= |w| <
//   13.5; what lies beyond is lumped into one bin at either end): 3200 counters of 16 bits.
//   The first-digit sums go to the unit's histogram as above; the counters of the 64
//   first-digit bins from 3 octaves below to 5 above the tile's mean |w| are written out as the
//   tile's record, with the bin of the tile's largest key, so that the unit's P99 can be
//   refined to the last bit without reading W again; the count of |w| < 1e-6 is a sum of counters.
// MASKED: salient weights (Sec. 3.5) marked in A.mask take no part: they are left out of
// the group statistics, and in every error sum their activation scale counts as zero.
// rot spreads an uneven number of clip passes over the four SIMDs from tile to tile.
template <int DT, bool MASKED, int MODE>
__device__ __forceinline__ void fit_score_tile(const FitScoreArgs& B, const FitScoreMat& A, const TileCoord& tc,
                                               const int rot, char* __restrict__ smem) {
    constexpr bool ONLY8 = MODE == FS_ONLY8;
    constexpr bool FEAT = MODE == FS_SCORE_FEAT || MODE == FS_FEAT_ONLY;
    constexpr bool SCORE = MODE != FS_FEAT_ONLY;
    static_assert(!(FEAT && MASKED), "the features are those of all the unit's weights");
    const int32_t G = A.g.chunk_w;
    constexpr int EB = Elem<DT>::bytes;
    const int32_t row_bytes = G * EB + 16;
    char* __restrict__ tile = smem;
    float* __restrict__ scol = reinterpret_cast<float*>(smem + TILE_ROWS * row_bytes);
    const int32_t mstride = mask_row_stride(G);
    constexpr int NROW = fs_nrow(MASKED);          // row of the scratch; its last three columns: ternary / binary / reference
    constexpr int ACC3_COL = NROW - 3;
    float2* __restrict__ gstat = reinterpret_cast<float2*>(scol + G + FS_WAVES * 16 * NROW);   // [FS_WAVES][TILE_ROWS] (min, max)
    float* __restrict__ sshort = reinterpret_cast<float*>(gstat + FS_WAVES * TILE_ROWS);   // s_c, 0 for the listed columns
    int32_t* __restrict__ hlist = reinterpret_cast<int32_t*>(sshort + G);   // the listed columns
    double* __restrict__ s1tab = reinterpret_cast<double*>(hlist + FS_HMAX);   // [FS_WAVES][TILE_ROWS] sum |w| of a quarter
    uint16_t* __restrict__ nktab = reinterpret_cast<uint16_t*>(s1tab + FS_WAVES * TILE_ROWS);   // kept weights of a quarter (masked): <= 128
    uint8_t* __restrict__ mtile = reinterpret_cast<uint8_t*>(nktab + (MASKED ? FS_WAVES * TILE_ROWS : 0));
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: lives in a scalar register

    // the features' LDS histogram, over the rows' scratch: fp32 inputs, the first radix digit
    // (FEAT_BINS 16-bit counters); bf16 inputs, FEAT_FINE_NCOARSE first-digit bins key by key
    // (FEAT_FINE_PAIRS dwords of two 16-bit counters: even key low, odd key high)
    constexpr bool FINE = FEAT && DT == WINDQ_BF16;
    constexpr int LH_DWORDS = FINE ? FEAT_FINE_PAIRS : FEAT_BINS / 2;
    uint32_t* __restrict__ lhist = reinterpret_cast<uint32_t*>(scol + G);
    static_assert(!FEAT || FS_WAVES * 16 * NROW * sizeof(float) >= LH_DWORDS * sizeof(uint32_t), "histogram fits the scratch");
    // Everything around the clip sweeps waits a lot (loads, barriers, cross-lane chains, the parameters'
    // divisions) and issues little: it runs at a raised wave priority, so that it is over sooner and the
    // SIMD's other wavefronts, in their sweeps, lose only the few issue slots it needs (1.2 % faster).
    __builtin_amdgcn_s_setprio(3);
    load_tile_raw<DT, 2>(A.W, A.g.ld, tc, G, tile);      // 256 threads: four pieces each, two loads in flight at a time
    for (int32_t c = threadIdx.x; c < G; c += FS_THREADS) scol[c] = A.s[tc.col0 + c];
    if (MASKED) load_mask_tile(A.mask, A.mask_ld, tc, G, mtile);
    if (FEAT) {
        for (int32_t b = threadIdx.x; b < LH_DWORDS; b += FS_THREADS) lhist[b] = 0u;
    }
    // Column selection for the 8-bit candidate, prepared per chunk (fit_score_prepare_kernel): s_c
    // of the columns on the short route (0 for the listed ones) and the list lie next to each
    // other, in the record as in LDS.
    int32_t nh = -1;           // listed columns; -1: no list, every column takes the exact route
    float s4_over_s2 = 0.0f;   // sum s_c^4 / sum s_c^2 over the short route: scales the tile's noise term
    if (SCORE && !ONLY8) {
        const float* __restrict__ rec = A.colsel + (size_t)(tc.col0 / G) * (size_t)colsel_words(G);
        for (int32_t c = threadIdx.x; c < G + FS_HMAX; c += FS_THREADS) sshort[c] = rec[c];
        // (wave-uniform: parked in scalar registers across the hot loops)
        nh = __builtin_amdgcn_readfirstlane(__float_as_int(rec[G + FS_HMAX]));
        s4_over_s2 = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(rec[G + FS_HMAX + 1])));
    }
    __syncthreads();

    // Group statistics (of the kept weights), once per tile: each wavefront scans a quarter of
    // the chunk's 8-column runs for all 64 rows -- minimum, maximum, and the sum of |w| in fp64
    // in column order -- and the quarters are combined through LDS, in order.
    const int32_t runs = G >> 3;
    const int32_t qc0 = ((wave * runs) >> 2) << 3, qc1 = (((wave + 1) * runs) >> 2) << 3;   // this wavefront's columns
    float f_sw = 0.0f, f_sw2 = 0.0f, f_cnt = 0.0f;     // features: this lane's row over this wavefront's columns
    double f_sabs = 0.0;
    {
        const int lane_s = fresh_lane();
        const char* __restrict__ wr = tile + lane_s * row_bytes;
        const uint8_t* __restrict__ mr = mtile + lane_s * mstride;
        const bool valid = lane_s < tc.nrows;             // rows past the unit's end are zeros, not weights
        float mn = INFINITY, mx = -INFINITY;
        double S1 = 0.0;
        int32_t nk = 0;
        for (int32_t c = qc0; c < qc1; c += 8) {
            float w[8];
            read8<DT>(wr, c, w);
            const uint32_t m = MASKED ? (uint32_t)mr[c >> 3] : 0u;
            if (MASKED && !ONLY8) nk += 8 - __builtin_popcount(m);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool kept = !MASKED || ((m >> j) & 1u) == 0u;
                mn = fminf(mn, kept ? w[j] : INFINITY);
                mx = fmaxf(mx, kept ? w[j] : -INFINITY);
                if (!ONLY8) S1 += kept ? (double)fabsf(w[j]) : 0.0;
            }
            if (FEAT) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    f_sw += w[j];
                    f_sw2 = fmaf(w[j], w[j], f_sw2);
                }
            }
            if (FINE) {
                // key = bits 16..30 of the pattern; its pair (key >> 1) is dword pair - 8 * FEAT_FINE_COARSE0
                // of the histogram, clamped: everything below the resolved range lands in the first
                // dword, everything above in the last.  Bit 16 picks the half.
                if (valid) {
                    char* __restrict__ lh = reinterpret_cast<char*>(lhist);
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const uint32_t bits = __float_as_uint(w[j]);
                        int32_t off = (int32_t)((bits >> 15) & 0xFFFCu) - 32 * FEAT_FINE_COARSE0;
                        off = min(max(off, 0), 4 * (FEAT_FINE_PAIRS - 1));
                        atomicAdd(reinterpret_cast<uint32_t*>(lh + off), max(bits & 0x10000u, 1u));
                    }
                }
            } else if (FEAT) {
                // bin of |w| = bits 20..30 of the pattern: dword (bin & 1023) of the LDS histogram, half
                // (bin >> 10).  The upper half is |w| >= 2: rare, so the wavefront asks once per eight
                // columns whether any of its rows needs it.
                uint32_t any_bits = 0u;
#pragma unroll
                for (int j = 0; j < 8; ++j) any_bits |= __float_as_uint(w[j]);
                if (valid) {
                    char* __restrict__ lh = reinterpret_cast<char*>(lhist);
                    if (__builtin_amdgcn_ballot_w64((any_bits & 0x40000000u) != 0u) == 0) {
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            atomicAdd(reinterpret_cast<uint32_t*>(lh + ((__float_as_uint(w[j]) >> 18) & 0xFFCu)), 1u);
                    } else {
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const uint32_t bits = __float_as_uint(w[j]);
                            atomicAdd(reinterpret_cast<uint32_t*>(lh + ((bits >> 18) & 0xFFCu)), 1u << ((bits >> 26) & 16u));
                        }
                    }
                }
            }
        }
        gstat[wave * TILE_ROWS + lane_s] = make_float2(mn, mx);
        if (!ONLY8) {
            s1tab[wave * TILE_ROWS + lane_s] = S1;
            if (MASKED) nktab[wave * TILE_ROWS + lane_s] = (uint16_t)nk;
        }
        if (FEAT) f_sabs = S1;
        __syncthreads();
    }

    float* __restrict__ red = scol + G + wave * 16 * NROW;

    // What a wavefront needs of the tile's rows as a whole, from the quarters' row minima, maxima and
    // sums (every wavefront takes all 4 x 64 of them, in the same order, so none waits for another):
    // does one row hold most of the rows' squared ranges (rows past the unit's end are zeros)?  For
    // the record of the feature pass, the tile's largest |w| and the sum of |w| (it only places the
    // record: fp32 will do).
    bool rows_even = true;
    float tile_amax = 0.0f, tile_sabs = 0.0f;
    if (FINE || (SCORE && !ONLY8 && nh >= 0)) {
        const int lane_t = fresh_lane();
        float mn = INFINITY, mx = -INFINITY, sabs = 0.0f;
#pragma unroll
        for (int q = 0; q < FS_WAVES; ++q) {
            const float2 st = gstat[q * TILE_ROWS + lane_t];
            mn = fminf(mn, st.x);
            mx = fmaxf(mx, st.y);
            if (FINE) sabs += (float)s1tab[q * TILE_ROWS + lane_t];
        }
        if (mn > mx) mn = mx = 0.0f;      // no weight of the group is kept
        const float rg = mx - mn;
        float sums[FINE ? 2 : 1], maxes[FINE ? 2 : 1];
        sums[0] = maxes[0] = rg * rg;
        if (FINE) {
            sums[1] = sabs;
            maxes[1] = fmaxf(fabsf(mn), fabsf(mx));
        }
        wave_sums_maxes(sums, maxes);
        rows_even = maxes[0] * ROW_SHARE <= sums[0];
        if (FINE) {
            tile_sabs = sums[1];
            tile_amax = maxes[1];
        }
    }

    if (FINE) {
        // (every counter at most 8192: the halves never carry)
        // The record covers the FEAT_WIN first-digit bins that end 5 octaves above the mean: P99
        // and half of it lie 0.7-2.7 octaves above the mean |w| of Gaussian to heavy-tailed
        // weights, wherever single outliers sit.
        const int lane_a = fresh_lane();
        const float mean = tile_sabs * __builtin_amdgcn_rcpf((float)(tc.nrows * G));
        const int32_t tmax = (int32_t)(__float_as_uint(tile_amax) >> 20);               // first-digit bin of the largest key
        const int32_t ct = (int32_t)(__float_as_uint(mean) >> 20) + 40;               // top bin of the record
        // first-digit sums into the unit's histogram: bin FEAT_FINE_COARSE0 + b is dwords 8b .. 8b+7
        uint32_t* __restrict__ gh = A.fhist + (size_t)tc.u * FEAT_BINS;
        if (threadIdx.x < FEAT_FINE_NCOARSE) {
            uint32_t sum = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t v = lhist[threadIdx.x * 8 + i];
                sum += (v & 0xffffu) + (v >> 16);
            }
            if (sum != 0u) atomicAdd(&gh[FEAT_FINE_COARSE0 + threadIdx.x], sum);
        }
        // the record: the FEAT_WIN first-digit bins that end at ct, key by key
        const size_t tidx = (size_t)tc.u * (size_t)A.g.tiles_per_unit + (size_t)tc.t;
        uint32_t* __restrict__ rec = A.ffine + tidx * (FEAT_WIN * 8);
        for (int32_t i = threadIdx.x; i < FEAT_WIN * 8; i += FS_THREADS) {
            const int32_t b = ct - (FEAT_WIN - 1) + (i >> 3) - FEAT_FINE_COARSE0;      // resolved bins: 1 .. NCOARSE - 2
            rec[i] = b >= 1 && b <= FEAT_FINE_NCOARSE - 2 ? lhist[b * 8 + (i & 7)] : 0u;
        }
        if (threadIdx.x == 0) A.fanchor[tidx] = (uint32_t)ct | ((uint32_t)tmax << 16);
        // |w| < 1e-6: the keys below sparse_key (inside the resolved range, above the first lumping bin)
        if (wave == 0) {
            const int32_t nlow = (int32_t)A.sparse_key - 16 * FEAT_FINE_COARSE0;      // counters below the threshold
            uint32_t cnt = 0;
            for (int32_t d = lane_a; 2 * d < nlow; d += 64) {
                const uint32_t v = lhist[d];
                cnt += (v & 0xffffu) + (2 * d + 1 < nlow ? v >> 16 : 0u);
            }
            f_cnt = (float)cnt;
        }
        __syncthreads();        // the scratch is free for the sums from here on
    } else if (FEAT) {
        // the tile's histogram into the unit's (every bin at most 8192: the halves never carry)
        uint32_t* __restrict__ gh = A.fhist + (size_t)tc.u * FEAT_BINS;
        const uint32_t thr_bin = (__float_as_uint(A.sparse_thr) >> 20) & 1023u;      // 1e-6 lies far below 2: lower half
        int tiny = 0;           // does the tile hold a weight at or below the bin of 1e-6?
        for (int32_t b = threadIdx.x; b < FEAT_BINS / 2; b += FS_THREADS) {
            const uint32_t v = lhist[b];
            if ((v & 0xffffu) != 0u) {
                atomicAdd(&gh[b], v & 0xffffu);
                tiny |= (uint32_t)b <= thr_bin ? 1 : 0;
            }
            if ((v >> 16) != 0u) atomicAdd(&gh[b + FEAT_BINS / 2], v >> 16);
        }
        tiny = __syncthreads_or(tiny);          // also: the scratch is free for the sums from here on
        if (tiny) {
            // count |w| < 1e-6 exactly: only tiles that hold such small weights pay for it
            const int lane_c = fresh_lane();
            const char* __restrict__ wr = tile + lane_c * row_bytes;
            uint32_t cnt = 0;
            for (int32_t c = qc0; c < qc1; c += 8) {
                float w[8];
                read8<DT>(wr, c, w);
#pragma unroll
                for (int j = 0; j < 8; ++j) cnt += fabsf(w[j]) < A.sparse_thr ? 1u : 0u;
            }
            f_cnt = lane_c < tc.nrows ? (float)cnt : 0.0f;
        }
    }
    // The tile's sums over rows wait in the scratch (columns FS_NRED ..) for the first clip pass,
    // whose sums they are collected with; a wavefront without a pass collects them by themselves.
    const size_t tile_index = (size_t)tc.u * (size_t)A.g.tiles_per_unit + (size_t)tc.t;
    if (FEAT) {
        const int lane_f = fresh_lane();
        // sum |w| stays fp64: lanes through the wavefront's scratch, four at a time, then sixteen, in order
        double* __restrict__ dred = reinterpret_cast<double*>(red);
        dred[lane_f] = f_sabs;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        double q4 = 0.0;
        if (lane_f < 16) q4 = ((dred[4 * lane_f] + dred[4 * lane_f + 1]) + dred[4 * lane_f + 2]) + dred[4 * lane_f + 3];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
        if (lane_f < 16) dred[64 + lane_f] = q4;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        if (lane_f == 3) {
            double tot = 0.0;
#pragma unroll
            for (int i = 0; i < 16; ++i) tot += dred[64 + i];
            A.fmoments[(tile_index * FEAT_QUARTERS + (size_t)wave) * 4 + 2] = tot;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
        const float v3[3] = {f_sw, f_sw2, f_cnt};
        rows_deposit<NROW>(v3, red, lane_f, FS_NRED);
    }
    // what lane FS_NRED + j of a collecting wavefront does with the tile's sum j
    // (the lane's part of an address as an unsigned 32-bit byte offset from a wave-uniform base: a
    // 64-bit index would have its upper half carried, as a register of zeros, across the hot loops)
    auto store_extra = [&](int lane, double tot) {
        const uint32_t j = (uint32_t)(lane - FS_NRED);
        if (FEAT && j < 3u) {
            char* base = reinterpret_cast<char*>(A.fmoments + (tile_index * FEAT_QUARTERS + (size_t)wave) * 4);
            *reinterpret_cast<double*>(base + (j == 2u ? 24u : j * 8u)) = tot;
        }
        const uint32_t j3 = (uint32_t)(lane - ACC3_COL);
        if (SCORE && !ONLY8 && j3 < 3u) {
            char* base = reinterpret_cast<char*>(A.partial + tile_index * (size_t)fit_score_ncand(B.K) + 4 * B.K + 3 * wave);
            *reinterpret_cast<double*>(base + j3 * 8u) = tot;
        }
    };
    if (!SCORE) {
        const int lane_f = fresh_lane();
        store_extra(lane_f, rows_collect<NROW>(red, lane_f, NROW));
        return;
    }

    const int32_t K = B.K;
    double* __restrict__ out = A.partial + tile_index * (size_t)fit_score_ncand(K);

    // Ternary absmean, binary sign*mean|w| and the reference energy: every wavefront scores
    // its quarter of the columns.  gamma = alpha = fp32(S1 / n), S1 = the quarters' sums of |w|
    // added in order (exact for bf16 inputs; for fp32 inputs it can differ from the strict
    // column-order sum in the last bit of the fp64, which the conversion to fp32 hides but for
    // ~1e-8 of the groups, and there by one ulp of gamma).
    if (!ONLY8) {
        const int lane_w = fresh_lane();
        const char* __restrict__ wrow = tile + lane_w * row_bytes;
        const uint8_t* __restrict__ mrow = mtile + lane_w * mstride;
        double S1 = 0.0;
        int32_t n_kept = MASKED ? 0 : G;
#pragma unroll
        for (int q = 0; q < FS_WAVES; ++q) {
            S1 += s1tab[q * TILE_ROWS + lane_w];
            if (MASKED) n_kept += (int32_t)nktab[q * TILE_ROWS + lane_w];
        }
        // n is the chunk width unless weights are masked out; the product with its reciprocal (from
        // the host) rounds to the same fp32 as the quotient, but for ~1e-9 of groups when G is not 2^k
        const float fam = MASKED ? (n_kept > 0 ? (float)(S1 / (double)n_kept) : 0.0f) : (float)(S1 * B.inv_G);
        const bool ok = fam >= FLT_MIN;
        // Fast-issue fp32 only, as in the clip passes.  y = clamp01(w/(2 gamma) + 1/2) maps
        // w/gamma in [-1, 1] onto [0, 1]; rne(2y) = q + 1 in {0, 1, 2} needs no clamp.
        const float gam = pin_vgpr(ok ? fam : 0.0f);
        const float ngam = pin_vgpr(ok ? -fam : 0.0f);
        const float hginv = pin_vgpr(ok ? 0.5f * __builtin_amdgcn_rcpf(fam) : 0.0f);
        const float nalpha = pin_vgpr(-fam);
        const float half = pin_vgpr(0.5f), two = pin_vgpr(2.0f);
        const float M = pin_vgpr(RNE_POS);
        float acc3[3] = {0.0f, 0.0f, 0.0f};
        for (int32_t c = qc0; c < qc1; c += 8) {
            float w[8];
            read8<DT>(wrow, c, w);
            const float4 sa = *reinterpret_cast<const float4*>(scol + c);
            const float4 sb = *reinterpret_cast<const float4*>(scol + c + 4);
            float s8[8] = {sa.x, sa.y, sa.z, sa.w, sb.x, sb.y, sb.z, sb.w};
            if (MASKED) {
                const uint32_t m = mrow[c >> 3];
                drop_masked(s8, m);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float sc = s8[j];
                const float y = fma_clamp01(w[j], hginv, half);
                const float qp = fmaf(y, two, M) - M;                    // q + 1
                const float rt = fmaf(qp, ngam, w[j] + gam) * sc;        // s_c (w - q gamma)
                acc3[0] = fmaf(rt, rt, acc3[0]);
                const float aw = __uint_as_float(__float_as_uint(w[j]) & 0x7fffffffu);
                const float rb = (aw + nalpha) * sc;                     // s_c (|w| - alpha)
                acc3[1] = fmaf(rb, rb, acc3[1]);
                const float w1 = w[j] * sc;
                acc3[2] = fmaf(w1, w1, acc3[2]);
            }
        }
        const int lane_r = fresh_lane();
        if (lane_r >= tc.nrows) acc3[0] = acc3[1] = acc3[2] = 0.0f;
        rows_deposit<NROW>(acc3, red, lane_r, ACC3_COL);
    }
    int32_t ncollect = ONLY8 ? FS_NRED : NROW;         // columns the next collection takes

    // The clip grid: n_kpass passes over FS_KB clip ratios each.  Pass i goes to wavefront
    // (i + rot) % 4.
    for (int item = (wave - rot) & (FS_WAVES - 1); item < B.n_kpass; item += FS_WAVES) {
        // The hot loop below needs every register the occupancy target allows.  The lane index
        // is therefore re-read from the hardware where it is needed (before the loop for the
        // row address, after it for the reduction) rather than kept alive across the loop,
        // which would spill it, and everything derived from it, to scratch memory.
        {
            float mn = INFINITY, mx = -INFINITY;
            const int lane_w = fresh_lane();
#pragma unroll
            for (int q = 0; q < FS_WAVES; ++q) {
                const float2 st = gstat[q * TILE_ROWS + lane_w];
                mn = fminf(mn, st.x);
                mx = fmaxf(mx, st.y);
            }
            if (mn > mx) mn = mx = 0.0f;      // no weight of the group is kept
            // zero inside the closed range of every group of the wavefront?
            const bool anchored = __builtin_amdgcn_ballot_w64(!(mn <= 0.0f && mx >= 0.0f)) == 0;
            KParams P[FS_KB];
            float acc[FS_KB][4];
#pragma unroll
            for (int i = 0; i < FS_KB; ++i) {
                int k = item * FS_KB + i;
                k = k < K ? k : K - 1;
                const float p = B.grid.p[k];
                const float flo = p * mn;
                const float fhi = p * mx;
                const float frg = fhi - flo;
                const float rinv = frg >= FLT_MIN ? __builtin_amdgcn_rcpf(frg) : 0.0f;
                float d8 = 0.0f;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    // step = range / (2^b - 1): the fp64 product rounds to the correctly rounded
                    // fp32 quotient (but for ~1e-9 of inputs, where it is one ulp off)
                    const double rq = b == 0 ? 1.0 / 255.0 : (b == 1 ? 1.0 / 15.0 : (b == 2 ? 1.0 / 7.0 : 1.0 / 3.0));
                    float d = (float)((double)frg * rq);
                    d = d >= FLT_MIN ? d : 0.0f;
                    if (b == 0) d8 = d;
                    if (!ONLY8 || b == 0) P[i].nd[b] = pin_vgpr(-d);
                    acc[i][b] = 0.0f;
                }
                // anchor: the 8-bit grid point nearest zero when zero lies inside the range, else lo
                float q0 = 0.0f;
                if (flo <= 0.0f && fhi >= 0.0f) q0 = __builtin_amdgcn_fmed3f(__builtin_rintf(-flo * rinv * 255.0f), 0.0f, 255.0f);
                const float c = fmaf(q0, d8, flo);
                P[i].rinv = rinv;
                P[i].h = pin_vgpr((anchored ? -flo : c - flo) * rinv);
                P[i].nc = pin_vgpr(-c);
                P[i].Mq = pin_vgpr(RNE_POS + q0);
                if (!ONLY8) P[i].nlo = pin_vgpr(-flo);
            }
            const float Q[4] = {pin_vgpr(255.0f), pin_vgpr(15.0f), pin_vgpr(7.0f), pin_vgpr(3.0f)};
            const float M = pin_vgpr(RNE_POS);
            const float nM = pin_vgpr(-RNE_POS);
            float nz[FS_KB];     // the noise terms of the short route (zero on the exact ones)
#pragma unroll
            for (int i = 0; i < FS_KB; ++i) nz[i] = 0.0f;
            // (the row addresses are formed from a fresh lane index in front of each sweep: kept
            // from here they would be spilled across the parameter set-up)
            __builtin_amdgcn_s_setprio(0);       // the sweeps: issue-bound, ordinary priority
            auto sweep = [&](auto anchored_t, auto normative_t) {
                constexpr bool AN = decltype(anchored_t)::value, NORM = decltype(normative_t)::value;
                if (NORM) {         // the 8-bit decision by the normative steps: 1/step in h's place
#pragma unroll
                    for (int i = 0; i < FS_KB; ++i) {
                        const float d8 = -P[i].nd[0];
                        P[i].h = pin_vgpr(d8 >= FLT_MIN ? 1.0f / d8 : 0.0f);
                        if (ONLY8) {        // (-lo is not kept through the set-up in this mode)
                            int k = item * FS_KB + i;
                            k = k < K ? k : K - 1;
                            P[i].nlo = pin_vgpr(-(B.grid.p[k] * mn));
                        }
                    }
                }
                const int lane_v = fresh_lane();
                const char* __restrict__ wrow = tile + lane_v * row_bytes;
                const uint8_t* __restrict__ mrow = mtile + lane_v * mstride;
                if (ONLY8) {
                    for (int32_t c = 0; c < G; c += 8) {
                        float w[8];
                        read8<DT>(wrow, c, w);
                        const float4 sa = *reinterpret_cast<const float4*>(scol + c);
                        const float4 sb = *reinterpret_cast<const float4*>(scol + c + 4);
                        float s8[8] = {sa.x, sa.y, sa.z, sa.w, sb.x, sb.y, sb.z, sb.w};
                        if (MASKED) {
                            const uint32_t m = mrow[c >> 3];
                            drop_masked(s8, m);
                        }
#pragma unroll
                        for (int j = 0; j < 8; ++j) score_weight_8<AN, NORM>(w[j], s8[j], P, Q[0], M, acc);
                    }
                } else {
                    for (int32_t c = 0; c < G; c += 4) {
                        float w[4];
                        read4<DT>(wrow, c, w);
                        const float4 sa = *reinterpret_cast<const float4*>(scol + c);
                        float s4[4] = {sa.x, sa.y, sa.z, sa.w};
                        if (MASKED) {
                            const uint32_t m = (uint32_t)mrow[c >> 3] >> (c & 4);
                            s4[0] = drop_if_set<0>(s4[0], m); s4[1] = drop_if_set<1>(s4[1], m);
                            s4[2] = drop_if_set<2>(s4[2], m); s4[3] = drop_if_set<3>(s4[3], m);
                        }
#pragma unroll
                        for (int j = 0; j < 4; ++j) score_weight_staged<AN, NORM>(w[j], s4[j], P, Q, M, nM, acc);
                    }
                }
            };
            // A sweep over every column takes the 8-bit rounding decision as the normative steps do when the
            // unit has few rows: there a single weight near a rounding tie can hold enough of the unit's error
            // for the neighbouring code's residual (the same magnitude to 4e-5) to show; it costs 7 %.
            const bool few_rows = A.g.R_u < FS_FEW_ROWS;
            if (!anchored) {
                if (few_rows) sweep(std::false_type{}, std::true_type{});
                else sweep(std::false_type{}, std::false_type{});
            } else if (ONLY8 || nh < 0 || !rows_even) {
                if (few_rows) sweep(std::true_type{}, std::true_type{});
                else sweep(std::true_type{}, std::false_type{});
            } else {
                const int lane_v = fresh_lane();
                const char* __restrict__ wrow = tile + lane_v * row_bytes;
                const uint8_t* __restrict__ mrow = mtile + lane_v * mstride;
                for (int32_t c = 0; c < G; c += 8) {
                    float w[8];
                    read8<DT>(wrow, c, w);
                    const float4 sa = *reinterpret_cast<const float4*>(sshort + c);
                    const float4 sb = *reinterpret_cast<const float4*>(sshort + c + 4);
                    float s8[8] = {sa.x, sa.y, sa.z, sa.w, sb.x, sb.y, sb.z, sb.w};
                    if (MASKED) {
                        const uint32_t m = mrow[c >> 3];
                        drop_masked(s8, m);
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j) score_weight_short(w[j], s8[j], P, Q, M, nM, acc);
                }
                // range^2 * (the lane's short-route 8-bit sum); range = 255 * step
#pragma unroll
                for (int i = 0; i < FS_KB; ++i) nz[i] = acc[i][0] * (P[i].nd[0] * P[i].nd[0]) * 65025.0f;
                for (int32_t hi = 0; hi < nh; ++hi) {
                    const int32_t c = __builtin_amdgcn_readfirstlane(hlist[hi]);
                    const float w = read1<DT>(wrow, c);
                    float sc = scol[c];
                    if (MASKED) sc = ((mrow[c >> 3] >> (c & 7)) & 1u) != 0u ? 0.0f : sc;
                    score_weight<true>(w, sc, P, Q, M, nM, acc);
                }
            }
            __builtin_amdgcn_s_setprio(3);
            float flat[FS_NRED];
#pragma unroll
            for (int i = 0; i < FS_KB; ++i) {
#pragma unroll
                for (int b = 0; b < 4; ++b) flat[i * 4 + b] = acc[i][b];
                flat[FS_KB * 4 + i] = nz[i];
            }
            const int lane_r = fresh_lane();
            if (lane_r >= tc.nrows) {
#pragma unroll
                for (int j = 0; j < FS_NRED; ++j) flat[j] = 0.0f;
            }
            rows_deposit<NROW>(flat, red, lane_r, 0);
            const double tot = rows_collect<NROW>(red, lane_r, ncollect);
            if (!ONLY8 && ncollect > FS_NRED) store_extra(lane_r, tot);
            ncollect = FS_NRED;
            if (lane_r < FS_KB * 4) {
                const int k = item * FS_KB + (lane_r >> 2);
                if (k < K && (!ONLY8 || (lane_r & 3) == 0)) out[(lane_r & 3) * K + k] = tot;
            } else if (lane_r < FS_NRED) {
                const int k = item * FS_KB + (lane_r - FS_KB * 4);
                if (k < K) {
                    float ratio = s4_over_s2;
                    asm volatile("" : "+s"(ratio));      // converted here, not ahead of the loops
                    out[fit_score_noise_slot(K) + k] = tot * (double)ratio;
                }
            }
        }
    }
    if (!ONLY8 && ncollect > FS_NRED) {     // no clip pass fell to this wavefront
        const int lane_r = fresh_lane();
        store_extra(lane_r, rows_collect<NROW>(red, lane_r, NROW));
    }
}

// What a scoring call sets up before its tiles run, per matrix: the column selection of every
// chunk, one wavefront each; the empty list of units for the exact 8-bit pass; and, with the
// unit features riding along, their counters at zero.
//   Column selection for the 8-bit candidate: a column whose s_c^2 exceeds tau times the chunk's
//   mean carries much of a unit's error by itself.  Such columns are listed and scored on the
//   exact route, one at a time; all others go down the short route, and their
//   S4/S2 = sum s_c^4 / sum s_c^2 scales a tile's noise term.  It depends on s alone, so the
//   chunk's tiles read it instead of deriving it again.
__global__ __launch_bounds__(FS_THREADS) void fit_score_prepare_kernel(const FitScoreArgs B) {
    const int mi = batch_index(B.prep_start, B.n, blockIdx.x);
    const FitScoreMat& A = B.m[mi];
    const int64_t local = (int64_t)blockIdx.x - B.prep_start[mi];
    const int64_t sel_groups = (A.g.n_chunks + FS_PREP_CHUNKS - 1) / FS_PREP_CHUNKS;
    if (local >= sel_groups) {
        const int64_t i = ((local - sel_groups) * FS_THREADS + (int64_t)threadIdx.x) * 4;
        if (i < A.fclear_words) *reinterpret_cast<uint4*>(A.fclear + i) = make_uint4(0u, 0u, 0u, 0u);
        if (i == 0 && A.flist_count != nullptr) *A.flist_count = 0u;
        return;
    }
    if (local == 0 && threadIdx.x == 0) *A.redo_count = 0u;      // the list the finalize kernel fills
    const int64_t j = local * FS_PREP_CHUNKS + (int64_t)(threadIdx.x >> 6);
    if (j >= A.g.n_chunks) return;
    const int l = threadIdx.x & 63;
    const int32_t G = A.g.chunk_w;
    const float* __restrict__ scol = A.s + j * G;
    float* __restrict__ sshort = A.colsel + (size_t)j * (size_t)colsel_words(G);    // s_c, 0 for the listed columns
    int32_t* __restrict__ hlist = reinterpret_cast<int32_t*>(sshort + G);            // the listed columns
    float ss = 0.0f;
    for (int32_t c = l; c < G; c += 64) {
        const float sv = scol[c];
        ss = fmaf(sv, sv, ss);
    }
    // below tau = 1 (never a positive tau) nothing is listed short: the threshold 0 lists every column with s_c != 0
    const float thr = A.tau * wave_sum_f32(ss) / (float)G;
    int32_t nh = 0;
    float t2 = 0.0f, t4 = 0.0f;
    for (int32_t blk = 0; blk < G; blk += 64) {
        const int32_t c = blk + l;
        const float sv = c < G ? scol[c] : 0.0f;
        const float s2 = sv * sv;
        const bool hv = s2 > thr;
        const uint64_t bal = __builtin_amdgcn_ballot_w64(hv);
        if (c < G) sshort[c] = hv ? 0.0f : sv;
        if (!hv) {
            t2 += s2;
            t4 = fmaf(s2, s2, t4);
        }
        const int32_t pos = nh + __builtin_popcountll(bal & ((1ull << l) - 1ull));
        if (hv && pos < FS_HMAX) hlist[pos] = c;
        nh += __builtin_popcountll(bal);
    }
    const float S2 = wave_sum_f32(t2), S4 = wave_sum_f32(t4);
    if (nh * 8 > G || !(A.tau > 0.0f)) nh = -1;      // so many that one exact sweep over all columns is cheaper
    if (l == 0) {
        hlist[FS_HMAX] = nh;
        sshort[G + FS_HMAX + 1] = S2 >= FLT_MIN ? S4 / S2 : 0.0f;
    }
}

template <int DT, bool MASKED, int MODE>
__global__ __launch_bounds__(FS_THREADS, 5) void fit_score_kernel(const FitScoreArgs B) {
    extern __shared__ char smem[];
    const int mi = batch_index(B.tile_start, B.n, blockIdx.x);
    const FitScoreMat& A = B.m[mi];
    const int64_t local = (int64_t)blockIdx.x - B.tile_start[mi];
    const TileCoord tc = tile_coord(A.g, local);
    fit_score_tile<DT, MASKED, MODE>(B, A, tc, blockIdx.x & (FS_WAVES - 1), smem);
}

// The tiles of the listed units once more, 8-bit candidates only, exact route.  A fixed grid
// walks the list; with nothing listed every workgroup ends after reading the counters.
template <int DT, bool MASKED>
__global__ __launch_bounds__(FS_THREADS, 5) void fit_score_redo_kernel(const FitScoreArgs B) {
    extern __shared__ char smem[];
    // (no table of the matrices' first tiles: indexed by a run-time value it would live in scratch memory)
    auto listed_tiles = [&](int i) -> int64_t {
        int64_t cnt = (int64_t)*B.m[i].redo_count;
        cnt = cnt < B.m[i].g.U ? cnt : B.m[i].g.U;
        return cnt * B.m[i].g.tiles_per_unit;
    };
    int64_t total = 0;
    for (int i = 0; i < B.n; ++i) total += listed_tiles(i);
    for (int64_t w = blockIdx.x; w < total; w += gridDim.x) {
        int mi = 0;
        int64_t first = 0;
        for (; mi + 1 < B.n; ++mi) {
            const int64_t nt = listed_tiles(mi);
            if (w < first + nt) break;
            first += nt;
        }
        const FitScoreMat& A = B.m[mi];
        const int64_t local = w - first;
        const int64_t li = local / A.g.tiles_per_unit;
        const int64_t u = A.redo_list[li];
        const TileCoord tc = tile_coord_of_unit(A.g, u, local - li * A.g.tiles_per_unit);
        fit_score_tile<DT, MASKED, FS_ONLY8>(B, A, tc, (int)(w & (FS_WAVES - 1)), smem);
        __syncthreads();      // the next tile overwrites this one's LDS
    }
}

// Per unit: add the tiles' partial errors in a fixed order, pick the clip index with the
// least error for each uniform bit-width (ties to the largest index), emit fp32.
// REDO = false: every unit; a unit whose 8-bit error may hold too much of the short route's
// rounding noise (see NOISE_MAX) is put on the list.  REDO = true: the listed units only,
// after their 8-bit partials have been replaced.
constexpr int FIN_THREADS = 1024;
constexpr int FIN_PHASES = FIN_THREADS / 64;
template <bool REDO>
__global__ __launch_bounds__(FIN_THREADS) void fit_score_finalize_kernel(const FitScoreArgs B) {
    __shared__ double part[FIN_PHASES][5 * WINDQ_MAX_CLIP + 12];
    __shared__ double E[5 * WINDQ_MAX_CLIP + 12];
    const int mi = batch_index(B.unit_start, B.n, blockIdx.x);
    const FitScoreMat& A = B.m[mi];
    int64_t u = (int64_t)blockIdx.x - B.unit_start[mi];
    if (REDO) {
        if (u >= (int64_t)*A.redo_count) return;
        u = A.redo_list[u];
    }
    const int32_t K = B.K;
    const int64_t tiles_per_unit = A.g.tiles_per_unit;
    float* __restrict__ err = A.err;
    uint8_t* __restrict__ clip_idx = A.clip_idx;
    float* __restrict__ ref_energy = A.ref_energy;
    const int32_t ncand = fit_score_ncand(K);
    const double* base = A.partial + (size_t)u * (size_t)tiles_per_unit * (size_t)ncand;
    const int phase = threadIdx.x >> 6;
    // phase p adds tiles p, p+16, p+32, ... in order; the 16 phase sums are then added in order
    for (int32_t cand = threadIdx.x & 63; cand < ncand; cand += 64) {
        double acc = 0.0;
#pragma unroll 4
        for (int64_t t = phase; t < tiles_per_unit; t += FIN_PHASES) acc += base[(size_t)t * ncand + cand];
        part[phase][cand] = acc;
    }
    __syncthreads();
    for (int32_t cand = threadIdx.x; cand < ncand; cand += FIN_THREADS) {
        double acc = 0.0;
#pragma unroll
        for (int p = 0; p < FIN_PHASES; ++p) acc += part[p][cand];
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
        if (!REDO && tid == 0 && E[fit_score_noise_slot(K) + bk] * NOISE_C1 > best * best) {
            const uint32_t pos = atomicAdd(A.redo_count, 1u);
            A.redo_list[pos] = (uint32_t)u;
        }
    } else if (tid < 7) {
        // ternary, binary, reference energy: the four column quarters, in order
        const int j = tid - 4;
        const double e = ((E[4 * K + j] + E[4 * K + 3 + j]) + E[4 * K + 6 + j]) + E[4 * K + 9 + j];
        if (j < 2) err[u * WINDQ_N_ERR + 4 + j] = (float)e;
        else if (ref_energy != nullptr) ref_energy[u] = (float)e;
    }
}

}  // namespace windq

using namespace windq;

// One matrix of a launch as the entry points see it.
struct FitItem {
    const windq_mat* W;
    const float* s;
    const uint8_t* mask;
    float* err;
    uint8_t* clip_idx;
    float* ref_energy;
    void* ws;
    size_t ws_bytes;
};

template <int MODE>
static int launch_tiles_untimed(const FitScoreArgs& A, int32_t dtype, bool masked, size_t lds, dim3 grid, hipStream_t hs);

// Profiling aid (windq_kernel_timer): while switched on, every launch of the main fit+score kernel is
// bracketed by a pair of HIP events on the launch stream.  Off by default; the only state the library keeps.
namespace {
struct KernelTimer {
    std::mutex mu;
    bool on = false;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pairs;
} g_ktimer;

void ktimer_drop_locked() {
    for (auto& p : g_ktimer.pairs) {
        (void)hipEventDestroy(p.first);
        (void)hipEventDestroy(p.second);
    }
    g_ktimer.pairs.clear();
}
}  // namespace

template <int MODE>
static int launch_tiles(const FitScoreArgs& A, int32_t dtype, bool masked, size_t lds, dim3 grid, hipStream_t hs) {
    std::unique_lock<std::mutex> lock(g_ktimer.mu);
    const bool timed = g_ktimer.on && MODE != FS_FEAT_ONLY;
    lock.unlock();
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (timed && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)) return WINDQ_EHIP;
    if (timed && hipEventRecord(e0, hs) != hipSuccess) return WINDQ_EHIP;
    const int st = launch_tiles_untimed<MODE>(A, dtype, masked, lds, grid, hs);
    if (timed) {
        if (hipEventRecord(e1, hs) != hipSuccess) return WINDQ_EHIP;
        lock.lock();
        g_ktimer.pairs.emplace_back(e0, e1);
    }
    return st;
}

template <int MODE>
static int launch_tiles_untimed(const FitScoreArgs& A, int32_t dtype, bool masked, size_t lds, dim3 grid, hipStream_t hs) {
    auto launch = [&](auto kernel) -> int {
        const int e = ensure_lds(reinterpret_cast<const void*>(kernel), lds);
        if (e != WINDQ_OK) return e;
        hipLaunchKernelGGL(kernel, grid, dim3(FS_THREADS), lds, hs, A);
        return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
    };
    constexpr bool CAN_MASK = MODE == FS_SCORE;
    if (dtype == WINDQ_BF16) {
        if (CAN_MASK && masked) return launch(&fit_score_kernel<WINDQ_BF16, CAN_MASK, MODE>);
        return launch(&fit_score_kernel<WINDQ_BF16, false, MODE>);
    }
    if (CAN_MASK && masked) return launch(&fit_score_kernel<WINDQ_F32, CAN_MASK, MODE>);
    return launch(&fit_score_kernel<WINDQ_F32, false, MODE>);
}

// feat: nullptr, or the filled feature batch of the same matrices: the main kernel then also makes the
// first pass of the unit features, and the feature kernels that follow it are launched from here.
static int fit_score_launch(const FitItem* items, int32_t n, int32_t chunk_w, int64_t unit_rows, const float* clip_grid,
                            int32_t K, const FeatBatch* feat, void* stream) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    int st = check_clip_grid(clip_grid, K);
    if (st != WINDQ_OK) return st;
    FitScoreArgs A;
    A.n = n;
    A.K = K;
    A.n_kpass = (K + FS_KB - 1) / FS_KB;
    A.inv_G = 1.0 / (double)chunk_w;
    for (int k = 0; k < WINDQ_MAX_CLIP; ++k) A.grid.p[k] = clip_grid[k < K ? k : K - 1];
    const bool masked = items[0].mask != nullptr;
    if (masked && feat != nullptr) return WINDQ_EINVAL;
    int64_t tiles = 0, units = 0, preps = 0;
    for (int32_t i = 0; i < n; ++i) {
        const FitItem& it = items[i];
        FitScoreMat& M = A.m[i];
        if (it.W == nullptr) return WINDQ_EINVAL;
        st = make_geometry(it.W, chunk_w, unit_rows, &M.g);
        if (st != WINDQ_OK) return st;
        if (it.s == nullptr || it.err == nullptr || it.clip_idx == nullptr) return WINDQ_EINVAL;
        if (it.W->dtype != items[0].W->dtype || (it.mask != nullptr) != masked) return WINDQ_EINVAL;   // one kernel per launch
        const FitScoreLayout L = fit_score_layout(M.g, K);
        if (it.ws == nullptr || it.ws_bytes < L.total || !aligned(it.ws, 256)) return WINDQ_EWORKSPACE;
        M.W = it.W->data;
        M.s = it.s;
        M.mask = it.mask;
        M.mask_ld = it.W->cols / 8;
        char* base = static_cast<char*>(it.ws);
        M.partial = reinterpret_cast<double*>(base + L.partial);
        M.redo_count = reinterpret_cast<uint32_t*>(base + L.redo_count);
        M.redo_list = reinterpret_cast<uint32_t*>(base + L.redo_list);
        M.colsel = reinterpret_cast<float*>(base + L.colsel);
        M.err = it.err;
        M.clip_idx = it.clip_idx;
        M.ref_energy = it.ref_energy;
        M.fmoments = feat != nullptr ? feat->m[i].moments : nullptr;
        M.fhist = feat != nullptr ? feat->m[i].hist : nullptr;
        M.ffine = feat != nullptr ? feat->m[i].fine : nullptr;
        M.fanchor = feat != nullptr ? feat->m[i].anchor : nullptr;
        M.sparse_thr = feat != nullptr ? feat->m[i].sparse_thr : 0.0f;
        M.sparse_key = feat != nullptr ? feat->m[i].sparse_key : 0u;
        M.fclear = M.fhist;
        M.fclear_words = feat != nullptr ? (feat->dtype == WINDQ_BF16 ? 1 : 3) * (int64_t)FEAT_BINS * M.g.U : 0;
        M.flist_count = feat != nullptr && feat->dtype == WINDQ_BF16 ? feat->m[i].list_count : nullptr;
        // tau: with the error spread evenly over R_u rows, listing the columns above tau times the
        // mean keeps the short route's noise in the unit's 8-bit error near 1e-6 (one standard
        // deviation; what the rows really do is measured per unit, see NOISE_MAX).  Below
        // tau = 1 every column takes the exact route.
        const float t = 7e-5f * (float)chunk_w * (float)M.g.R_u;
        M.tau = t < 1.0f ? 0.0f : t;
        A.tile_start[i] = tiles;
        A.unit_start[i] = units;
        A.prep_start[i] = preps;
        tiles += M.g.n_tiles;
        units += M.g.U;
        preps += (M.g.n_chunks + FS_PREP_CHUNKS - 1) / FS_PREP_CHUNKS + (M.fclear_words + FS_PREP_CLEAR - 1) / FS_PREP_CLEAR;
    }
    for (int32_t i = n; i <= WINDQ_MAX_BATCH; ++i) {
        A.tile_start[i] = tiles;
        A.unit_start[i] = units;
        A.prep_start[i] = preps;
    }
    for (int32_t i = n; i < WINDQ_MAX_BATCH; ++i) A.m[i] = A.m[0];
    if (tiles > (int64_t)0x7fffffff || preps > (int64_t)0x7fffffff) return WINDQ_ESHAPE;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int32_t dtype = items[0].W->dtype;
    const size_t lds = fit_score_lds_bytes(dtype, chunk_w, masked);
    const dim3 grid((unsigned)tiles);
    hipLaunchKernelGGL(fit_score_prepare_kernel, dim3((unsigned)preps), dim3(FS_THREADS), 0, hs, A);
    if (hipPeekAtLastError() != hipSuccess) return WINDQ_EHIP;
    if (feat != nullptr) {
        st = launch_tiles<FS_SCORE_FEAT>(A, dtype, false, lds, grid, hs);
    } else {
        st = launch_tiles<FS_SCORE>(A, dtype, masked, lds, grid, hs);
    }
    if (st != WINDQ_OK) return st;
    hipLaunchKernelGGL(fit_score_finalize_kernel<false>, dim3((unsigned)units), dim3(FIN_THREADS), 0, hs, A);
    if (hipPeekAtLastError() != hipSuccess) return WINDQ_EHIP;
    // the units the finalize kernel listed: their 8-bit candidates on the exact route, finalized again
    const dim3 redo_grid((unsigned)(tiles < FS_REDO_GRID ? tiles : FS_REDO_GRID));
    auto launch_redo = [&](auto kernel) -> int {
        const int e = ensure_lds(reinterpret_cast<const void*>(kernel), lds);
        if (e != WINDQ_OK) return e;
        hipLaunchKernelGGL(kernel, redo_grid, dim3(FS_THREADS), lds, hs, A);
        return hipPeekAtLastError() == hipSuccess ? WINDQ_OK : WINDQ_EHIP;
    };
    if (dtype == WINDQ_BF16) st = masked ? launch_redo(&fit_score_redo_kernel<WINDQ_BF16, true>) : launch_redo(&fit_score_redo_kernel<WINDQ_BF16, false>);
    else st = masked ? launch_redo(&fit_score_redo_kernel<WINDQ_F32, true>) : launch_redo(&fit_score_redo_kernel<WINDQ_F32, false>);
    if (st != WINDQ_OK) return st;
    hipLaunchKernelGGL(fit_score_finalize_kernel<true>, dim3((unsigned)units), dim3(FIN_THREADS), 0, hs, A);
    if (hipPeekAtLastError() != hipSuccess) return WINDQ_EHIP;
    if (feat != nullptr) return features_launch_rest(*feat, hs);
    return WINDQ_OK;
}

// The first pass of the unit features by itself (windq_unit_features): the same tile kernel, scoring nothing.
int windq::features_launch_tiles(const FeatBatch& F, hipStream_t hs) {
    FitScoreArgs A;
    A.n = F.n;
    A.K = 1;
    A.n_kpass = 0;
    A.inv_G = 0.0;
    for (int k = 0; k < WINDQ_MAX_CLIP; ++k) A.grid.p[k] = 1.0f;
    int64_t tiles = 0, units = 0;
    for (int32_t i = 0; i < WINDQ_MAX_BATCH; ++i) {
        const FeatArgs& f = F.m[i < F.n ? i : 0];
        FitScoreMat& M = A.m[i];
        M = FitScoreMat{};
        M.W = f.W;
        M.s = f.s;
        M.g = f.g;
        M.fmoments = f.moments;
        M.fhist = f.hist;
        M.ffine = f.fine;
        M.fanchor = f.anchor;
        M.sparse_thr = f.sparse_thr;
        M.sparse_key = f.sparse_key;
        if (i < F.n) {
            A.tile_start[i] = tiles;
            A.unit_start[i] = units;
            tiles += f.g.n_tiles;
            units += f.g.U;
        }
    }
    for (int32_t i = F.n; i <= WINDQ_MAX_BATCH; ++i) {
        A.tile_start[i] = tiles;
        A.unit_start[i] = units;
    }
    if (tiles > (int64_t)0x7fffffff) return WINDQ_ESHAPE;
    const size_t lds = fit_score_lds_bytes(F.dtype, F.m[0].g.chunk_w, false);
    return launch_tiles<FS_FEAT_ONLY>(A, F.dtype, false, lds, dim3((unsigned)tiles), hs);
}

static int fit_score_impl(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows, const uint8_t* mask,
                          const float* clip_grid, int32_t K, float* err, uint8_t* clip_idx, float* ref_energy,
                          void* ws, size_t ws_bytes, void* stream) {
    if (W == nullptr) return WINDQ_EINVAL;
    const FitItem it = {W, s, mask, err, clip_idx, ref_energy, ws, ws_bytes};
    return fit_score_launch(&it, 1, chunk_w, unit_rows, clip_grid, K, nullptr, stream);
}

extern "C" int windq_fit_score_all_bits(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows,
                                        const float* clip_grid, int32_t K, float* err, uint8_t* clip_idx,
                                        float* ref_energy, void* ws, size_t ws_bytes, void* stream) {
    return fit_score_impl(W, s, chunk_w, unit_rows, nullptr, clip_grid, K, err, clip_idx, ref_energy, ws, ws_bytes, stream);
}

extern "C" int windq_fit_score_all_bits_prot(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows,
                                             const uint8_t* mask, const float* clip_grid, int32_t K, float* err,
                                             uint8_t* clip_idx, float* ref_energy, void* ws, size_t ws_bytes,
                                             void* stream) {
    if (mask == nullptr) return WINDQ_EINVAL;
    return fit_score_impl(W, s, chunk_w, unit_rows, mask, clip_grid, K, err, clip_idx, ref_energy, ws, ws_bytes, stream);
}

extern "C" int windq_fit_score_all_bits_batch(const windq_fit_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows,
                                              const float* clip_grid, int32_t K, void* stream) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    FitItem its[WINDQ_MAX_BATCH];
    for (int32_t i = 0; i < n; ++i)
        its[i] = {items[i].W, items[i].s, items[i].mask, items[i].err, items[i].clip_idx, items[i].ref_energy, items[i].ws,
                  items[i].ws_bytes};
    return fit_score_launch(its, n, chunk_w, unit_rows, clip_grid, K, nullptr, stream);
}

// Features and fit+score from one read of W.  The workspace holds the features layout first, then fit+score's.
static int fused_launch(const windq_fused_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows, const float* clip_grid,
                        int32_t K, void* stream) {
    if (items == nullptr || n < 1 || n > WINDQ_MAX_BATCH) return WINDQ_EINVAL;
    if (K < 1 || K > WINDQ_MAX_CLIP) return WINDQ_EINVAL;
    FeatItem fi[WINDQ_MAX_BATCH];
    FitItem si[WINDQ_MAX_BATCH];
    for (int32_t i = 0; i < n; ++i) {
        const windq_fused_item& it = items[i];
        if (it.W == nullptr) return WINDQ_EINVAL;
        Geometry g;
        const int st = make_geometry(it.W, chunk_w, unit_rows, &g);
        if (st != WINDQ_OK) return st;
        const size_t fbytes = features_ws_bytes(g, it.W->dtype);
        if (it.ws == nullptr || it.ws_bytes < fbytes + fit_score_ws_bytes(g, K) || !aligned(it.ws, 256)) return WINDQ_EWORKSPACE;
        fi[i] = {it.W, it.s, it.feat, it.ws, fbytes};
        si[i] = {it.W, it.s, nullptr, it.err, it.clip_idx, it.ref_energy, static_cast<char*>(it.ws) + fbytes, it.ws_bytes - fbytes};
    }
    FeatBatch F;
    const int st = features_fill(fi, n, chunk_w, unit_rows, &F);
    if (st != WINDQ_OK) return st;
    return fit_score_launch(si, n, chunk_w, unit_rows, clip_grid, K, &F, stream);
}

extern "C" int windq_features_fit_score(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows,
                                        const float* clip_grid, int32_t K, float* feat, float* err, uint8_t* clip_idx,
                                        float* ref_energy, void* ws, size_t ws_bytes, void* stream) {
    const windq_fused_item it = {W, s, feat, err, clip_idx, ref_energy, ws, ws_bytes};
    return fused_launch(&it, 1, chunk_w, unit_rows, clip_grid, K, stream);
}

extern "C" int windq_features_fit_score_batch(const windq_fused_item* items, int32_t n, int32_t chunk_w, int64_t unit_rows,
                                              const float* clip_grid, int32_t K, void* stream) {
    return fused_launch(items, n, chunk_w, unit_rows, clip_grid, K, stream);
}

// Scratch memory of windq_fit_score_all_bits_static: the workspace of one call, held by every
// GPU the library runs on until the process ends.  In host code the array's name is only a
// stand-in: its device address is looked up once per device (below) and used from then on.
static __device__ __align__(256) unsigned char scratch[WINDQ_STATIC_SCRATCH_BYTES];

constexpr int STATIC_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[STATIC_MAX_DEVICES];      // per device, nullptr until looked up

// Device address of `scratch` on the current device.
static int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return WINDQ_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return WINDQ_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return WINDQ_OK;
}

extern "C" int windq_fit_score_all_bits_static(const windq_mat* W, const float* s, int32_t chunk_w, int64_t unit_rows,
                                               const float* clip_grid, int32_t K, float* err, uint8_t* clip_idx,
                                               float* ref_energy, void* stream) {
    if (W == nullptr) return WINDQ_EINVAL;
    int st = check_clip_grid(clip_grid, K);
    if (st != WINDQ_OK) return st;
    Geometry g;
    st = make_geometry(W, chunk_w, unit_rows, &g);
    if (st != WINDQ_OK) return st;
    if (fit_score_ws_bytes(g, K) > (size_t)WINDQ_STATIC_SCRATCH_BYTES) return WINDQ_EWORKSPACE;
    void* ptr = nullptr;
    st = static_scratch(&ptr);
    if (st != WINDQ_OK) return st;
    // Every slot of the workspace that a call reads is written by that call first (the kernels
    // clear the one counter themselves), so what the previous call left behind does not matter.
    return fit_score_impl(W, s, chunk_w, unit_rows, nullptr, clip_grid, K, err, clip_idx, ref_energy, ptr,
                          (size_t)WINDQ_STATIC_SCRATCH_BYTES, stream);
}

extern "C" int windq_kernel_timer(int32_t enable) {
    std::lock_guard<std::mutex> lock(g_ktimer.mu);
    ktimer_drop_locked();
    g_ktimer.on = enable != 0;
    return WINDQ_OK;
}

extern "C" int windq_kernel_timer_read(double* total_ms, int64_t* launches) {
    if (total_ms == nullptr || launches == nullptr) return WINDQ_EINVAL;
    std::lock_guard<std::mutex> lock(g_ktimer.mu);
    double sum = 0.0;
    for (auto& p : g_ktimer.pairs) {
        float ms = 0.0f;
        if (hipEventSynchronize(p.second) != hipSuccess || hipEventElapsedTime(&ms, p.first, p.second) != hipSuccess) {
            ktimer_drop_locked();
            return WINDQ_EHIP;
        }
        sum += (double)ms;
    }
    *total_ms = sum;
    *launches = (int64_t)g_ktimer.pairs.size();
    ktimer_drop_locked();
    return WINDQ_OK;
}

extern "C" int windq_fit_score_rescored_units(const void* ws, int32_t dtype, int64_t rows, int64_t cols, int32_t chunk_w,
                                              int64_t unit_rows, int32_t K, int64_t* n_units) {
    if (ws == nullptr || n_units == nullptr || K < 1 || K > WINDQ_MAX_CLIP) return WINDQ_EINVAL;
    windq_mat fake = {ws, dtype, 0, rows, cols, cols};      // shape checks only: the data pointer is not read
    Geometry g;
    const int st = make_geometry(&fake, chunk_w, unit_rows, &g);
    if (st != WINDQ_OK) return st;
    const FitScoreLayout L = fit_score_layout(g, K);
    uint32_t cnt = 0;
    if (hipMemcpy(&cnt, static_cast<const char*>(ws) + L.redo_count, sizeof(cnt), hipMemcpyDeviceToHost) != hipSuccess)
        return WINDQ_EHIP;
    *n_units = (int64_t)cnt;
    return WINDQ_OK;
}
