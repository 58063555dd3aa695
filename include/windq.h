/*
 * windq.h - C ABI of libwindq: the per-unit hot path of WINDQuant's allocation
 * method on one AMD MI355X (gfx950).
 *
 * The paper's controller assigns one of seven treatments (Eq. 3: skip/16, 8, 4, 3,
 * 2, 1.58, 1 bit) to every column-chunk unit of every linear weight matrix under a
 * global bit budget (Sec. 3.1, Eq. 1).  This library is the data-parallel work that
 * feeds it: calibration activation scales, the unit's state features (Table 1), the
 * fit of the lightweight quantizer at all six bit-widths scored by activation-aware
 * reconstruction error (Sec. 3.5, App. "Per-unit Scale Optimization"), packed codes
 * of a chosen plan, and effective-bit accounting (Eq. 5).
 *
 * Conventions shared by every call
 *   - W is [rows x cols] = [out features x in features], row major, leading
 *     dimension `ld` in elements.  A "column" is an input channel: the axis the
 *     activation scale s[cols] lives on.
 *   - chunk j  = columns [j*chunk_w, (j+1)*chunk_w).
 *     unit  u  = chunk j over `unit_rows` consecutive rows; unit_rows = 0 means all
 *                rows (the paper's unit).  u = row_block * n_chunks + j.
 *     group    = one row of a unit (chunk_w consecutive weights of one output row);
 *                g = u * R_u + local_row, R_u = rows per unit.  Scales are per group
 *                (App. "Per-unit Scale Optimization": per-group scales, group size =
 *                chunk size).
 *   - action index a in 0..6 follows Eq. 3: 0 skip(16), 1: 8, 2: 4, 3: 3, 4: 2,
 *     5: 1.58 (ternary), 6: 1 bit.
 *   - Pointers are DEVICE pointers unless the comment says HOST.  The caller owns
 *     every buffer, including the workspace `ws` (size from windq_workspace_bytes;
 *     256-byte aligned).  The library allocates nothing, frees nothing, never
 *     synchronises and keeps no state: all device work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and outputs are
 *     valid once that stream has reached the end of the call's work.
 *   - Every function returns a status.  All argument checks happen before the first
 *     launch: on any status other than WINDQ_OK / WINDQ_EHIP no output was touched.
 *   - Shape limits of the kernels: cols % chunk_w == 0, chunk_w % 8 == 0,
 *     8 <= chunk_w <= WINDQ_MAX_CHUNK, unit_rows == 0 or rows % unit_rows == 0,
 *     data pointers 16-byte aligned, ld % 8 == 0.
 */
#ifndef WINDQ_H
#define WINDQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum windq_status {
    WINDQ_OK = 0,
    WINDQ_EINVAL = 1,     /* null pointer, bad scalar, misaligned pointer            */
    WINDQ_ESHAPE = 2,     /* shape outside the limits listed above                   */
    WINDQ_EDTYPE = 3,     /* dtype is not one of windq_dtype                         */
    WINDQ_EWORKSPACE = 4, /* ws is NULL or smaller than windq_workspace_bytes says   */
    WINDQ_EHIP = 5        /* a launch failed; hipGetLastError() still holds the cause */
};

enum windq_dtype { WINDQ_F32 = 0, WINDQ_BF16 = 1 };

enum windq_call {
    WINDQ_CALL_CALIB_STATS = 0,
    WINDQ_CALL_UNIT_FEATURES = 1,
    WINDQ_CALL_FIT_SCORE = 2,
    WINDQ_CALL_APPLY_PLAN = 3,
    WINDQ_CALL_SALIENT = 4,       /* windq_salient_select and windq_salient_encode */
    WINDQ_CALL_UNIT_SALIENCY = 5,
    WINDQ_CALL_DEQUANT = 6,
    WINDQ_CALL_REFINE = 7,
    WINDQ_CALL_FEATURES_FIT_SCORE = 8,
    WINDQ_CALL_DEQUANT_GEMV = 9
};

#define WINDQ_N_ACTIONS 7
#define WINDQ_N_ERR 6        /* error columns: 8, 4, 3, 2, 1.58, 1 bit */
#define WINDQ_N_FEAT 8
#define WINDQ_MAX_CLIP 64    /* longest clip grid */
#define WINDQ_MAX_CHUNK 512  /* widest chunk */
#define WINDQ_MAX_BATCH 8    /* most matrices one *_batch call takes */
#define WINDQ_STATIC_SCRATCH_BYTES (8u << 20) /* workspace built into the library for windq_fit_score_all_bits_static */

/* A row-major matrix in device memory.  Never written by the library. */
typedef struct windq_mat {
    const void* data; /* DEVICE, 16-byte aligned */
    int32_t dtype;    /* windq_dtype */
    int32_t reserved; /* set to 0 */
    int64_t rows, cols;
    int64_t ld;       /* elements between consecutive rows, >= cols, multiple of 8 */
} windq_mat;

/*
 * Calibration statistics (App. "Salient Weight Protection": a per-channel activation
 * scale estimated in a calibration forward pass; Table 1 dims 9-11 are statistics of
 * it).  X is [tokens x channels].
 *   s_absmean[c] = mean_t |x_tc|          (the activation scale used everywhere else)
 *   s_rms[c]     = sqrt(mean_t x_tc^2)    (optional, may be NULL; its square is the
 *                                          diagonal of X^T X / tokens)
 * Sums are accumulated in fp64 in a fixed order (bit-reproducible run to run).
 */
int windq_calib_stats(const windq_mat* X, float* s_absmean /*[cols]*/, float* s_rms /*[cols] or NULL*/,
                      void* ws, size_t ws_bytes, void* stream);

/*
 * windq_calib_stats for up to WINDQ_MAX_BATCH activation matrices (a decoder block has four
 * distinct inputs) of one element type; those of at most 4096 tokens share ONE launch.  Item i
 * is one per-matrix call; results are the same bit for bit.  `items` is a HOST array read
 * during the call.
 */
typedef struct windq_calib_item {
    const windq_mat* X;     /* HOST descriptor of a device matrix [tokens][channels] */
    float* s_absmean;       /* [channels] */
    float* s_rms;           /* [channels] or NULL */
    void* ws;
    size_t ws_bytes;
} windq_calib_item;
int windq_calib_stats_batch(const windq_calib_item* items /*HOST [n]*/, int32_t n, void* stream);

/*
 * State features of every unit (Table 1, dims 0-4 and 9-11), feat[u][8] =
 *   mean, std (population), mean|w|, fraction with |w| < 1e-6,
 *   fraction with |w| > 0.5 * P99(|w|)  (P99 = nearest-rank order statistic, rank
 *   ceil(0.99 n), found exactly by radix selection),
 *   mean, std (population), max of s over the unit's chunk_w input channels.
 * Counts are exact integers; moments are accumulated in fp64.
 */
int windq_unit_features(const windq_mat* W, const float* s /*[cols]*/, int32_t chunk_w, int64_t unit_rows,
                        float* feat /*[U][8]*/, void* ws, size_t ws_bytes, void* stream);

/*
 * Fit the lightweight quantizer of every unit at all six bit-widths and score each fit
 * by the activation-aware reconstruction error  E = sum_rows sum_c s_c^2 (w - w_hat)^2
 * (Sec. 3.5: local scale fitting per unit, reconstruction error decides fallback; the
 * weighting uses the per-channel activation scale, the only activation statistic the
 * paper defines).  Per group, in fp32 with one correctly rounded operation per step:
 *   uniform b in {8,4,3,2} at clip ratio p:  lo = p*min, hi = p*max, step = (hi-lo)/(2^b-1),
 *       code = clamp(rne((w-lo) * (1/step)), 0, 2^b-1), w_hat = lo + code*step
 *       (step below the smallest normal fp32: step = 0, codes 0);
 *   ternary:  gamma = mean|w|, q = clamp(rne(w * (1/gamma)), -1, 1), w_hat = gamma*q;
 *   binary:   alpha = mean|w|, w_hat = alpha * (w >= 0 ? +1 : -1).
 * For each uniform bit-width the clip ratio is chosen once per unit: the grid index
 * with the least unit error, exact ties to the largest index.
 *   clip_grid  HOST [K], ascending, each in (0, 1], 1 <= K <= WINDQ_MAX_CLIP
 *   err        [U][6]  errors in the order 8, 4, 3, 2, 1.58, 1 bit (uniform ones at
 *                      their chosen clip index), raw weighted sums of squares
 *   clip_idx   [U][4]  chosen grid index for 8, 4, 3, 2 bit
 *   ref_energy [U] or NULL: sum s_c^2 w^2, to normalise err
 * Errors are accumulated in fp32 along a group and in fp64 beyond it, in a fixed order
 * (results are bit-reproducible run to run).  They agree with the definition above evaluated
 * in fp64 to ~1e-7 relative.  The 8-bit candidate has two arithmetic routes: an exact one
 * (~1e-7), and a shorter one whose fp32 roundings leave noise of random sign in the unit's
 * error.  The short route is used only where that noise is provably small for the data at
 * hand: columns that hold much of the chunk's sum of s_c^2, and tiles in which one row holds
 * most of the rows' squared ranges, take the exact route; and every unit's noise variance is
 * summed from its own per-row errors (each rounding taken at its largest possible size).  A
 * unit whose noise could exceed 3e-6 of its 8-bit error (one standard deviation; measured
 * deviations are ~0.4 of that estimate) has its 8-bit candidates scored again on the exact
 * route before the call's work ends, whatever the input.  |s_c * w| must square inside fp32's
 * normal range.
 *   That accuracy is a unit's, not a single weight's.  A weight's residual s_c (w - lo - code step)
 * comes from fp32-rounded products: an absolute error near 1e-7 s_c (hi - lo) at 4 bits and below
 * (1e-7 s_c step at 8 bits, exact route), and at 8 bits a weight within ~2e-5 steps of a rounding
 * tie may take the neighbouring code (a residual of the same magnitude to 4e-5; units of fewer
 * than 64 rows take that decision exactly as written above instead, at 7 % more time).  These
 * errors are random in sign from weight to weight and average out of a unit's sum once its error
 * is spread over a few dozen weights, as it is in the units of weight matrices (thousands of
 * rows).  Where ONE weight carries nearly all of a unit's error - a single-row "unit" with one
 * large activation scale; a row a thousand times its neighbours that meets a column forty times
 * its neighbours - the 4-, 3- and 2-bit errors have been seen 1e-5 to 1e-4 off.
 */
int windq_fit_score_all_bits(const windq_mat* W, const float* s /*[cols]*/, int32_t chunk_w, int64_t unit_rows,
                             const float* clip_grid /*HOST [K]*/, int32_t K,
                             float* err /*[U][6]*/, uint8_t* clip_idx /*[U][4]*/, float* ref_energy /*[U] or NULL*/,
                             void* ws, size_t ws_bytes, void* stream);

/*
 * windq_fit_score_all_bits for callers that can neither allocate device memory nor bring a
 * workspace: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The workspace is an array of WINDQ_STATIC_SCRATCH_BYTES built into the library's
 * device code (every GPU the process uses holds its own copy until the process ends); its device
 * address is looked up once per device, on the first call made with that device current.  The
 * call allocates and frees nothing.  Same arguments, outputs and results (bit for bit) as
 * windq_fit_score_all_bits without `ws`.
 *   WINDQ_EWORKSPACE  the shape needs more than WINDQ_STATIC_SCRATCH_BYTES (check beforehand with
 *                     windq_workspace_bytes(WINDQ_CALL_FIT_SCORE, ...)): nothing is launched.
 *                     The need is 8 (5K + 12) bytes per 64-row tile of a chunk plus 4 per unit:
 *                     4.9 MB for 4096 x 11008 or 11008 x 4096 at chunk 128, K = 20.
 *   WINDQ_EHIP        the address lookup failed.
 * All calls on one GPU share that GPU's array and it keeps the previous call's contents (every
 * slot a call reads it writes first): calls that overlap in time on one GPU - on different
 * streams, or from different threads - race.  Calls on one stream are ordered and safe.
 */
int windq_fit_score_all_bits_static(const windq_mat* W, const float* s /*[cols]*/, int32_t chunk_w, int64_t unit_rows,
                                    const float* clip_grid /*HOST [K]*/, int32_t K,
                                    float* err /*[U][6]*/, uint8_t* clip_idx /*[U][4]*/, float* ref_energy /*[U] or NULL*/,
                                    void* stream);

/*
 * Profiling aid for the dominant kernel.  windq_kernel_timer(1) switches it on: from then on every
 * launch of the main fit+score kernel (by any of the fit+score entry points, the fused ones included)
 * is bracketed by a pair of HIP events on the launch stream, so that the kernel's own duration can be
 * told apart from the small kernels that follow it in the same call.  windq_kernel_timer_read waits
 * for the recorded launches, returns the sum of their durations in milliseconds and their number, and
 * forgets them.  windq_kernel_timer(0) switches it off.  Off by default.  While it is on the library
 * creates events (host-side state, nothing on the device) and must not be used under graph capture;
 * windq_kernel_timer_read waits for the device.  HOST only.
 */
int windq_kernel_timer(int32_t enable);
int windq_kernel_timer_read(double* total_ms /*HOST*/, int64_t* launches /*HOST*/);

/*
 * Diagnostic: how many units of the last windq_fit_score_all_bits (or _prot, or batch item) call
 * that used workspace `ws` had their 8-bit candidates scored a second time on the exact route.
 * Pass the shape arguments of that call.  Unlike every other entry point this one copies a
 * counter to the host and therefore waits for the device: call it after the stream has finished.
 */
int windq_fit_score_rescored_units(const void* ws, int32_t dtype, int64_t rows, int64_t cols, int32_t chunk_w,
                                   int64_t unit_rows, int32_t K, int64_t* n_units /*HOST*/);

/*
 * windq_unit_features for up to WINDQ_MAX_BATCH matrices with one launch per pass instead of
 * one per pass and matrix (see windq_fit_score_all_bits_batch for the contract: item i is one
 * per-matrix call, results are the same bit for bit).
 */
/*
 * Diagnostic: how many units of the last windq_unit_features or windq_features_fit_score call (or
 * batch item) that used workspace `ws` needed the exact pass over their weights for P99 (bf16
 * inputs: units whose 99th percentile lies far from the bulk of one of their tiles, or outside
 * 2^-20 .. 13.5; always 0 for fp32 inputs).  Pass the shape arguments of that call.  Copies a
 * counter to the host and therefore waits for the device: call it after the stream has finished.
 */
int windq_unit_features_exact_units(const void* ws, int32_t dtype, int64_t rows, int64_t cols, int32_t chunk_w,
                                    int64_t unit_rows, int64_t* n_units /*HOST*/);

typedef struct windq_feat_item {
    const windq_mat* W;     /* HOST descriptor of a device matrix */
    const float* s;         /* [cols] */
    float* feat;            /* [U][8] */
    void* ws;
    size_t ws_bytes;
} windq_feat_item;
int windq_unit_features_batch(const windq_feat_item* items /*HOST [n]*/, int32_t n, int32_t chunk_w, int64_t unit_rows,
                              void* stream);

/*
 * windq_fit_score_all_bits for up to WINDQ_MAX_BATCH matrices with ONE launch of the scoring
 * kernel (and of each small kernel around it: one that prepares, per-unit sums, the second 8-bit
 * pass): the matrices of a decoder block are small against this GPU, and a launch per matrix
 * leaves it partly empty at every start and end.  Item i is one per-matrix call: the same
 * arguments, the same workspace size, and bit for bit the same results.  All items share chunk_w,
 * unit_rows, the clip grid and the element type.  `items` is a HOST array read during the call.
 * WINDQ_EINVAL for n outside 1..WINDQ_MAX_BATCH or mixed element types; otherwise as the
 * per-matrix call (nothing is launched if any item fails its checks).  With a protection mask in
 * every item this is the batch form of the *_prot call.
 */
typedef struct windq_fit_item {
    const windq_mat* W;     /* HOST descriptor of a device matrix */
    const float* s;         /* [cols] */
    const uint8_t* mask;    /* NULL, or [rows][cols/8] as in windq_fit_score_all_bits_prot: all items or none */
    float* err;             /* [U][6] */
    uint8_t* clip_idx;      /* [U][4] */
    float* ref_energy;      /* [U] or NULL */
    void* ws;
    size_t ws_bytes;
} windq_fit_item;
int windq_fit_score_all_bits_batch(const windq_fit_item* items /*HOST [n]*/, int32_t n, int32_t chunk_w,
                                   int64_t unit_rows, const float* clip_grid /*HOST [K]*/, int32_t K, void* stream);

/*
 * windq_unit_features and windq_fit_score_all_bits from ONE read of W (Table 1 and Sec. 3.5 are both
 * per-unit work on the same weights): the fit+score kernel, which holds every tile in LDS anyway,
 * also takes the moments, the count of |w| < 1e-6 and the histograms of |w| that decide P99 from it;
 * the small feature kernels that finish follow on the stream (bf16 inputs: W is not read again; a unit
 * whose P99 lies far from the bulk of one of its tiles gets an exact pass of its own).  Outputs are bit
 * for bit those of the two separate calls.  Workspace: windq_workspace_bytes(WINDQ_CALL_FEATURES_FIT_SCORE, ...).
 * The batch form is to this call what windq_fit_score_all_bits_batch is to the per-matrix one.
 */
int windq_features_fit_score(const windq_mat* W, const float* s /*[cols]*/, int32_t chunk_w, int64_t unit_rows,
                             const float* clip_grid /*HOST [K]*/, int32_t K,
                             float* feat /*[U][8]*/, float* err /*[U][6]*/, uint8_t* clip_idx /*[U][4]*/,
                             float* ref_energy /*[U] or NULL*/, void* ws, size_t ws_bytes, void* stream);
typedef struct windq_fused_item {
    const windq_mat* W;     /* HOST descriptor of a device matrix */
    const float* s;         /* [cols] */
    float* feat;            /* [U][8] */
    float* err;             /* [U][6] */
    uint8_t* clip_idx;      /* [U][4] */
    float* ref_energy;      /* [U] or NULL */
    void* ws;
    size_t ws_bytes;
} windq_fused_item;
int windq_features_fit_score_batch(const windq_fused_item* items /*HOST [n]*/, int32_t n, int32_t chunk_w,
                                   int64_t unit_rows, const float* clip_grid /*HOST [K]*/, int32_t K, void* stream);

/* Packed bytes of one group under an action: ceil(chunk_w*b/8), ceil(chunk_w/5) for
 * ternary, 0 for skip; -1 for an action outside 0..6 or chunk_w <= 0.  HOST only. */
int64_t windq_bytes_per_group(int32_t action, int32_t chunk_w);

/*
 * Byte offsets of the packed payload of every unit of a plan (HOST only, no GPU).
 * Unit u occupies [code_off[u], code_off[u] + R_u * bytes_per_group) and every
 * payload starts 16-byte aligned; code_off[U] is the stream length.
 * WINDQ_EINVAL if an action is outside 0..6.
 */
int windq_plan_layout(const uint8_t* action /*HOST [U]*/, int64_t n_units, int64_t rows_per_unit, int32_t chunk_w,
                      int64_t* code_off /*HOST [U+1]*/);

/*
 * Materialise a plan (Sec. 3.3: the environment applies the selected quantization to
 * the unit).  For every unit with action != skip, refit each group at that bit-width
 * with exactly the fp32 steps listed at windq_fit_score_all_bits, at clip ratio
 * clip_grid[clip_idx[u][a-1]] for uniform actions (p = 1 when clip_idx is NULL), and
 * write
 *   scale[g]   step / gamma / alpha           offset[g]  lo, or 0 for ternary and binary
 *   codes      per group, rows of a unit consecutive from code_off[u]:
 *              integer b: LSB-first bitstream (code i in bits [i*b, (i+1)*b));
 *              ternary: five trits (q+1) per byte, byte = sum trit_j 3^j, tail zero padded;
 *              the padding up to the next 16-byte boundary after a unit is zeroed.
 * Skip units write no codes and scale = offset = 0.  A unit whose action is outside
 * 0..6 or whose payload does not fit in [0, codes_bytes) is treated as skip (use
 * windq_plan_layout to build code_off).
 */
int windq_apply_plan(const windq_mat* W, int32_t chunk_w, int64_t unit_rows,
                     const uint8_t* action /*[U]*/, const uint8_t* clip_idx /*[U][4] or NULL*/,
                     const float* clip_grid /*HOST [K]*/, int32_t K,
                     const int64_t* code_off /*[U+1]*/, uint8_t* codes, size_t codes_bytes,
                     float* scale /*[U*R_u]*/, float* offset /*[U*R_u]*/,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * windq_apply_plan for up to WINDQ_MAX_BATCH matrices in one launch (see
 * windq_fit_score_all_bits_batch for the contract: item i is one per-matrix call with its own
 * plan, code stream and outputs; results are the same bit for bit).
 */
typedef struct windq_apply_item {
    const windq_mat* W;        /* HOST descriptor of a device matrix */
    const uint8_t* mask;       /* NULL, or as in windq_apply_plan_prot: all items or none */
    const uint8_t* action;     /* [U] */
    const uint8_t* clip_idx;   /* [U][4] or NULL */
    const int64_t* code_off;   /* [U+1] */
    uint8_t* codes;
    size_t codes_bytes;
    float* scale;              /* [U*R_u] */
    float* offset;             /* [U*R_u] */
    void* ws;
    size_t ws_bytes;
} windq_apply_item;
int windq_apply_plan_batch(const windq_apply_item* items /*HOST [n]*/, int32_t n, int32_t chunk_w, int64_t unit_rows,
                           const float* clip_grid /*HOST [K]*/, int32_t K, void* stream);

/*
 * Effective-bit accounting of a plan (Eq. 5), HOST only, exact integers:
 *   B_i = 16 n_i for skip, else b_i (n_i - n_i^p) + 8 n_i^p,
 * in centibits (bits x 100: 1600/800/400/300/200/158/100) so that 1.58 stays integral.
 * The average bit-width is total_centibits / (100 total_weights); the plan meets a
 * target b (Eq. 1) iff total_centibits <= 100 b total_weights.
 * WINDQ_EINVAL on an action outside 0..6, n < 0 or n_prot outside [0, n].
 */
int windq_effective_bits(const uint8_t* action /*HOST [U]*/, const int64_t* n_unit /*HOST [U]*/,
                         const int64_t* n_prot /*HOST [U] or NULL = 0*/, int64_t n_units,
                         int64_t* total_centibits /*HOST*/, int64_t* total_weights /*HOST*/);

/*
 * Salient-weight protection (Sec. 3.5; App. "Salient Weight Protection"): per unit, a
 * fraction of the weights, those with the largest saliency |w| * s_c, is kept out of the
 * low-bit quantizer and stored in INT8; Eq. 5 charges them 8 bits each.
 *
 * The rate is given in parts per million so that the count is an exact integer:
 * n_p = floor(n_unit * rate_ppm / 10^6) protected weights in every unit (the same for all
 * units of a matrix).  -1 if n_unit < 0 or rate_ppm > 10^6.  HOST only.
 */
int64_t windq_n_protected(int64_t n_unit, uint32_t rate_ppm);

/*
 * Select the protected set of every unit: its n_p weights of largest saliency
 * fp32(|w| * |s_c|) (one fp32 multiply), found exactly by radix selection; weights of
 * equal saliency are taken in the order of their flat index inside the unit
 * (local_row * chunk_w + column).
 *   mask  [rows][cols/8] bytes, dense: bit (c mod 8) of byte c/8 of a row is 1 where
 *         weight (row, c) is protected.  Every byte of it is written.
 * Needs rows_per_unit * chunk_w < 2^32.
 */
int windq_salient_select(const windq_mat* W, const float* s /*[cols]*/, int32_t chunk_w, int64_t unit_rows,
                         uint32_t rate_ppm, uint8_t* mask /*[rows][cols/8]*/,
                         void* ws, size_t ws_bytes, void* stream);

/*
 * Store the protected weights of a mask in INT8 (Sec. 3.5: "stored in INT8"), per unit:
 *   prot_scale[u] = sigma = fp32(max |w_p| / 127), 0 if below the smallest normal fp32
 *   prot_codes    [U][n_p] int8: clamp(rne(w * fp32(1/sigma)), -127, 127) of the unit's
 *                 protected weights in flat-index order (0 when sigma = 0)
 *   err_prot[u]   sum s_c^2 (w - code * sigma)^2 over them (fp64 sums, fixed order)
 * `mask` must hold exactly n_p bits per unit (as windq_salient_select writes it for the
 * same rate); surplus bits of a malformed mask are not stored.
 */
int windq_salient_encode(const windq_mat* W, const float* s /*[cols]*/, int32_t chunk_w, int64_t unit_rows,
                         const uint8_t* mask /*[rows][cols/8]*/, uint32_t rate_ppm,
                         int8_t* prot_codes /*[U][n_p]*/, float* prot_scale /*[U]*/, float* err_prot /*[U]*/,
                         void* ws, size_t ws_bytes, void* stream);

/*
 * windq_salient_select / windq_salient_encode for up to WINDQ_MAX_BATCH matrices with one
 * launch per kernel instead of one per kernel and matrix (a decoder block has seven
 * matrices: twelve launches to select, four to encode).  Results are bit-identical to the
 * per-matrix calls.  One chunk width, unit_rows, rate and element type for all items; every
 * item brings its own workspace (WINDQ_CALL_SALIENT for its shape).  select reads W, s and
 * writes mask; encode reads W, s, mask and writes prot_codes, prot_scale, err_prot (select
 * ignores those three).  All items are checked before the first launch; WINDQ_EINVAL for n
 * outside 1..WINDQ_MAX_BATCH or mixed element types, otherwise as the per-matrix calls.
 */
typedef struct windq_salient_item {
    const windq_mat* W;
    const float* s;           /* [cols] */
    uint8_t* mask;            /* [rows][cols/8]: select writes it, encode reads it */
    int8_t* prot_codes;       /* [U][n_p]   (encode) */
    float* prot_scale;        /* [U]        (encode) */
    float* err_prot;          /* [U]        (encode) */
    void* ws;
    size_t ws_bytes;
} windq_salient_item;
int windq_salient_select_batch(const windq_salient_item* items /*HOST [n]*/, int32_t n, int32_t chunk_w,
                               int64_t unit_rows, uint32_t rate_ppm, void* stream);
int windq_salient_encode_batch(const windq_salient_item* items /*HOST [n]*/, int32_t n, int32_t chunk_w,
                               int64_t unit_rows, uint32_t rate_ppm, void* stream);

/*
 * windq_fit_score_all_bits and windq_apply_plan under a protection mask (Sec. 3.5: the
 * remaining weights use the selected bit-width).  Protected weights take no part in the
 * fit: a group's min, max and mean |w| run over its kept weights (mean = sum / number
 * kept; a group with none kept has scale = offset = 0), and err / ref_energy sum over kept
 * weights only.  The code stream keeps its dense layout: the slot of a protected weight
 * holds 0.  Everything else is as in the unmasked calls; `mask` as written by
 * windq_salient_select, never NULL.  Workspaces as WINDQ_CALL_FIT_SCORE / _APPLY_PLAN.
 */
int windq_fit_score_all_bits_prot(const windq_mat* W, const float* s /*[cols]*/, int32_t chunk_w, int64_t unit_rows,
                                  const uint8_t* mask /*[rows][cols/8]*/,
                                  const float* clip_grid /*HOST [K]*/, int32_t K,
                                  float* err /*[U][6]*/, uint8_t* clip_idx /*[U][4]*/, float* ref_energy /*[U] or NULL*/,
                                  void* ws, size_t ws_bytes, void* stream);
int windq_apply_plan_prot(const windq_mat* W, int32_t chunk_w, int64_t unit_rows,
                          const uint8_t* mask /*[rows][cols/8]*/,
                          const uint8_t* action /*[U]*/, const uint8_t* clip_idx /*[U][4] or NULL*/,
                          const float* clip_grid /*HOST [K]*/, int32_t K,
                          const int64_t* code_off /*[U+1]*/, uint8_t* codes, size_t codes_bytes,
                          float* scale /*[U*R_u]*/, float* offset /*[U*R_u]*/,
                          void* ws, size_t ws_bytes, void* stream);

/*
 * The deterministic allocator the paper compares its controller with (App. "Comparison with
 * Heuristic Sensitivity Allocator"), and the fallback of Sec. 3.5.
 *
 * Saliency score of every unit: the mean of |w| * |s_c| over the unit (fp64 sums, fixed order).
 */
int windq_unit_saliency(const windq_mat* W, const float* s /*[cols]*/, int32_t chunk_w, int64_t unit_rows,
                        float* sal /*[U]*/, void* ws, size_t ws_bytes, void* stream);

/*
 * Greedy plan from saliency scores (HOST only, exact integers; uses temporary host memory).
 * Units are ranked by saliency, most salient first (equal scores: lower index first).
 * Every unit starts at 2 bits; the least salient floor(U * frac_1bit_ppm / 10^6) units are
 * pushed to 1 bit and the next floor(U * frac_ternary_ppm / 10^6) to 1.58; while the plan
 * exceeds target_centibits * sum(n_unit) under Eq. 5, units are demoted one level at a time
 * from the least salient upward (2 -> 1.58 in a first sweep, 1.58 -> 1 in a second); then
 * the most salient units are promoted 2 -> 3 wherever the budget permits, and after that
 * 3 -> 4 likewise.  *feasible = 0 if even the all-1-bit plan exceeds the budget.
 * WINDQ_EINVAL on a NaN score, n < 0, n_prot outside [0, n] or a fraction above 10^6.
 */
int windq_heuristic_plan(const float* sal /*HOST [U]*/, const int64_t* n_unit /*HOST [U]*/,
                         const int64_t* n_prot /*HOST [U] or NULL = 0*/, int64_t n_units,
                         int64_t target_centibits, uint32_t frac_1bit_ppm, uint32_t frac_ternary_ppm,
                         uint8_t* action /*HOST out [U]*/, int64_t* total_centibits /*HOST*/, int32_t* feasible /*HOST*/);

/*
 * Fallback to a higher-precision operator when the reconstruction error of the selected one
 * is excessive (Sec. 3.5), HOST only: while err[u][a-1] > max_rel_err * ref_energy[u] (compared
 * exactly), unit u climbs 1 -> 1.58 -> 2 -> 3 -> 4 -> 8 -> skip.  `action` is updated in place;
 * the caller re-checks the budget with windq_effective_bits.
 */
int windq_fallback_promote(uint8_t* action /*HOST in/out [U]*/, const float* err /*HOST [U][6]*/,
                           const float* ref_energy /*HOST [U]*/, int64_t n_units, float max_rel_err,
                           int64_t* n_changed /*HOST*/);

/*
 * The way back from the packed artefact (Sec. 3.5 scores a fit by its reconstruction error;
 * this recomputes that error from the stored codes, scales and offsets alone).  For every
 * unit of a plan as windq_apply_plan wrote it:
 *   uniform:  w_hat = offset + code * scale    ternary: scale * (trit - 1)    binary: +-scale
 *   err[u]    sum s_c^2 (w - w_hat)^2 with w_hat in fp64 from the stored fp32 numbers (what
 *             windq_fit_score_all_bits reported for that bit-width and clip index); 0 for skip
 *   w_hat     [rows][cols] fp32, dense: the reconstruction, one fused multiply-add per weight;
 *             skip units keep their weights
 * mask NULL or as in windq_apply_plan_prot: protected weights are left out of err and their
 * w_hat is 0 (their values live in the INT8 side stream).  err or w_hat may be NULL, not both.
 * Entries outside 0..6, at an offset that is not a multiple of 16 (windq_plan_layout makes none)
 * or pointing outside [0, codes_bytes) count as skip.
 */
int windq_dequant_plan(const windq_mat* W, const float* s /*[cols]*/, int32_t chunk_w, int64_t unit_rows,
                       const uint8_t* mask /*[rows][cols/8] or NULL*/, const uint8_t* action /*[U]*/,
                       const int64_t* code_off /*[U+1]*/, const uint8_t* codes, size_t codes_bytes,
                       const float* scale /*[U*R_u]*/, const float* offset /*[U*R_u]*/,
                       float* err /*[U] or NULL*/, float* w_hat /*[rows][cols] or NULL*/,
                       void* ws, size_t ws_bytes, void* stream);

/*
 * windq_dequant_plan for up to WINDQ_MAX_BATCH matrices in one launch (plus one that sums the
 * errors): bit-identical to the per-matrix calls.  One chunk width, unit_rows and element
 * type for all items; every item brings its own workspace (WINDQ_CALL_DEQUANT for its shape).
 * Matrices whose pointers or leading dimension are not 16-byte aligned take a second pair of
 * launches, as they take a slower kernel alone.
 */
typedef struct windq_dequant_item {
    const windq_mat* W;
    const float* s;           /* [cols] */
    const uint8_t* mask;      /* [rows][cols/8] or NULL */
    const uint8_t* action;    /* [U] */
    const int64_t* code_off;  /* [U+1] */
    const uint8_t* codes;
    size_t codes_bytes;
    const float* scale;       /* [U*R_u] */
    const float* offset;      /* [U*R_u] */
    float* err;               /* [U] or NULL */
    float* w_hat;             /* [rows][cols] or NULL */
    void* ws;
    size_t ws_bytes;
} windq_dequant_item;
int windq_dequant_plan_batch(const windq_dequant_item* items /*HOST [n]*/, int32_t n, int32_t chunk_w,
                             int64_t unit_rows, void* stream);

/*
 * The product of the reconstruction with a vector, from the packed artefact alone (the first piece of
 * a path that serves the quantized weights): for every row r
 *   y[r] = sum_c w_hat[r][c] * x[c],   w_hat as windq_dequant_plan reconstructs it (fp32, one fused
 *          multiply-add per weight; skip units keep their weights: W is read for them only;
 *          protected weights of a mask count as 0: their values live in the INT8 side stream).
 * Eight columns at a time are multiplied and summed in fp32 (fused multiply-adds in column order), those
 * runs in fp64 (a row's runs of one chunk, then the chunks in order), and y is rounded once: results are
 * bit-reproducible and differ from the exact product by at most ~1e-6 of sum_c |w_hat x|.
 *   x [cols] f32, y [rows] f32 (every element written).  Workspace: WINDQ_CALL_DEQUANT_GEMV.
 * Plan entries are checked as in windq_dequant_plan (a malformed one counts as skip).  The batch form
 * takes up to WINDQ_MAX_BATCH matrices (one chunk width, unit_rows, element type) in one launch plus
 * one that sums the chunks.
 */
int windq_dequant_gemv(const windq_mat* W, int32_t chunk_w, int64_t unit_rows,
                       const uint8_t* mask /*[rows][cols/8] or NULL*/, const uint8_t* action /*[U]*/,
                       const int64_t* code_off /*[U+1]*/, const uint8_t* codes, size_t codes_bytes,
                       const float* scale /*[U*R_u]*/, const float* offset /*[U*R_u]*/,
                       const float* x /*[cols]*/, float* y /*[rows]*/, void* ws, size_t ws_bytes, void* stream);
typedef struct windq_gemv_item {
    const windq_mat* W;
    const uint8_t* mask;      /* [rows][cols/8] or NULL */
    const uint8_t* action;    /* [U] */
    const int64_t* code_off;  /* [U+1] */
    const uint8_t* codes;
    size_t codes_bytes;
    const float* scale;       /* [U*R_u] */
    const float* offset;      /* [U*R_u] */
    const float* x;           /* [cols] */
    float* y;                 /* [rows] */
    void* ws;
    size_t ws_bytes;
} windq_gemv_item;
int windq_dequant_gemv_batch(const windq_gemv_item* items /*HOST [n]*/, int32_t n, int32_t chunk_w,
                             int64_t unit_rows, void* stream);

/*
 * windq_apply_plan with refined scales (App. "Per-unit Scale Optimization": each operator fits
 * its scale by a short local optimisation of the reconstruction loss on the unit).  Every
 * group is seeded with its grid fit (clip ratio clip_grid[clip_idx[u][a-1]], p = 1 when
 * clip_idx is NULL) and refined for n_iter (0..64) rounds of
 *     codes by the fp32 steps of windq_fit_score_all_bits  |  closed-form activation-weighted
 *     least squares: uniform (offset, step) from the 2x2 normal equations of
 *     min sum s_c^2 (w - offset - code * step)^2; ternary gamma = sum s_c^2 q w / sum s_c^2 q^2;
 *     binary (signs fixed, one solve when n_iter >= 1) alpha = sum s_c^2 |w| / sum s_c^2.
 * Sums are fp64 in column order, parameters are rounded to fp32 after every solve; a round
 * whose problem is singular or whose step would be below the smallest normal fp32 ends the
 * refinement of that group.  Outputs as windq_apply_plan, plus
 *   err [U]   the activation-weighted error of the refined plan (0 for skip units).
 * mask NULL or as in windq_apply_plan_prot.  n_iter = 0 reproduces windq_apply_plan.
 */
int windq_refine_plan(const windq_mat* W, const float* s /*[cols]*/, int32_t chunk_w, int64_t unit_rows,
                      const uint8_t* mask /*[rows][cols/8] or NULL*/,
                      const uint8_t* action /*[U]*/, const uint8_t* clip_idx /*[U][4] or NULL*/,
                      const float* clip_grid /*HOST [K]*/, int32_t K, int32_t n_iter,
                      const int64_t* code_off /*[U+1]*/, uint8_t* codes, size_t codes_bytes,
                      float* scale /*[U*R_u]*/, float* offset /*[U*R_u]*/, float* err /*[U]*/,
                      void* ws, size_t ws_bytes, void* stream);

/*
 * windq_refine_plan for up to WINDQ_MAX_BATCH matrices in one launch (plus one that sums the
 * errors): bit-identical to the per-matrix calls.  One chunk width, unit_rows, clip grid,
 * round count and element type for all items; masks and clip indices may be NULL item by
 * item; every item brings its own workspace (WINDQ_CALL_REFINE for its shape).
 */
typedef struct windq_refine_item {
    const windq_mat* W;
    const float* s;           /* [cols] */
    const uint8_t* mask;      /* [rows][cols/8] or NULL */
    const uint8_t* action;    /* [U] */
    const uint8_t* clip_idx;  /* [U][4] or NULL */
    const int64_t* code_off;  /* [U+1] */
    uint8_t* codes;
    size_t codes_bytes;
    float* scale;             /* [U*R_u] */
    float* offset;            /* [U*R_u] */
    float* err;               /* [U] */
    void* ws;
    size_t ws_bytes;
} windq_refine_item;
int windq_refine_plan_batch(const windq_refine_item* items /*HOST [n]*/, int32_t n, int32_t chunk_w, int64_t unit_rows,
                            const float* clip_grid /*HOST [K]*/, int32_t K, int32_t n_iter, void* stream);

/* Workspace bytes a call needs for these shapes (0 if the shape is invalid). HOST only. */
size_t windq_workspace_bytes(int32_t which_call, int32_t dtype, int64_t rows, int64_t cols,
                             int32_t chunk_w, int64_t unit_rows, int32_t K);

const char* windq_status_str(int status);

#ifdef __cplusplus
}
#endif
#endif /* WINDQ_H */
