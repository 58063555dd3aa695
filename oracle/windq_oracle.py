"""CPU oracle for the per-unit hot path of WINDQuant's allocation method.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check and
the benchmark's cpu_baseline leg may import it.  It shares no code with the HIP
library and never calls it.  It is written to be checked against the paper by eye:
plain numpy, one step per line, no blocking, no fusion.  Floating point is fp64
unless a line is marked [N] ("normative fp32"): those steps define stored fp32
quantities (scales, offsets) and integer codes, and are evaluated with IEEE fp32
operations, one correctly rounded operation per step, so that any conforming
implementation reproduces them bit for bit.

What the paper fixes and where:
  * units are column chunks of a weight matrix (Sec. 3.1, "Problem Definition");
  * the action set {16 (skip), 8, 4, 3, 2, 1.58, 1} in that order (Eq. 3);
  * state features 0-4 and 9-11 (Table 1);
  * activation scale = per input channel statistic of calibration activations,
    saliency = |w| * scale (Sec. 3.5 and App. "Salient Weight Protection");
  * quantizers fit "per group", group size = chunk size (App. "Per-unit Scale
    Optimization");
  * effective-bit accounting B_i and the average b-bar (Eq. 5).
What the paper leaves open (the loss, the scale fit, clipping, rounding, packing)
follows the deterministic closed-form / grid-search restatement of the method:
uniform k-bit scale+offset with a clip grid, ternary absmean, binary sign*mean|w|,
scored by the activation-weighted squared error  sum_c a_c (w - w_hat)^2  with
a_c = s_c^2 (a diagonal weighting: the only activation statistic the paper defines
is per channel, so no Gram matrix appears).

Conventions.  W is [R_out x C_in] row major; "column" = input channel.  Chunk j is
columns [j*G, (j+1)*G).  A unit is chunk j over `unit_rows` consecutive rows
(unit_rows = 0: all rows, the paper's definition).  Unit index u = row_block *
n_chunks + j.  A group is one row of a unit (G consecutive weights of one output
row); group index g = u * R_u + local_row.  Inputs are float32 ndarrays holding the
exact input values (bf16 inputs are passed widened, which is exact).

Beyond the five hot-path calls the module holds, to the same rules: salient-weight
protection (Sec. 3.5 and App. "Salient Weight Protection": exact top-n_p selection,
protection mask, masked fits and plans, INT8 storage), the heuristic sensitivity
allocator and the fallback to higher precision (App. "Comparison with Heuristic
Sensitivity Allocator", Sec. 3.5), iterative scale refinement (App. "Per-unit Scale
Optimization") and the dequantisation of a packed plan.

Parity pins (tests/test_oracle_*.py): closed forms, brute force on tiny groups,
hand-computed examples, a library least-squares solve, and golden bytes.  Not pinned
by anything: whether these deterministic fits reproduce the paper's learned LSQ/SEQ
scales or its perplexities, and whether the allocator's two knobs match the paper's
unstated thresholds ("parity unpinned": no weights, code or corpus exist to compare
against).
"""
from __future__ import annotations

import math

import numpy as np

f32 = np.float32
f64 = np.float64

# Eq. 3: action index -> bit-width.  Centibits make 1.58 an integer.
ACTIONS = ("skip", "8", "4", "3", "2", "1.58", "1")
ACTION_CENTIBITS = (1600, 800, 400, 300, 200, 158, 100)
UNIFORM_BITS = (8, 4, 3, 2)          # order of the err / clip_idx columns
N_ERR = 6                            # 8, 4, 3, 2, 1.58, 1
FLT_MIN_NORMAL = f32(2.0 ** -126)    # below this a step size counts as degenerate


# --------------------------------------------------------------------------- units
def unit_shape(R: int, C: int, G: int, unit_rows: int = 0):
    """(n_row_blocks, n_chunks, R_u).  Sec. 3.1: units are column chunks."""
    if G <= 0 or R <= 0 or C <= 0:
        raise ValueError("empty matrix or chunk")
    if C % G != 0:
        raise ValueError("cols must be a multiple of the chunk width")
    R_u = R if unit_rows == 0 else unit_rows
    if R % R_u != 0:
        raise ValueError("unit_rows must divide rows")
    return R // R_u, C // G, R_u


def unit_view(W: np.ndarray, G: int, unit_rows: int, u: int) -> np.ndarray:
    """The [R_u x G] block of weights that is unit u."""
    n_rb, n_chunks, R_u = unit_shape(W.shape[0], W.shape[1], G, unit_rows)
    rb, j = divmod(u, n_chunks)
    return W[rb * R_u:(rb + 1) * R_u, j * G:(j + 1) * G]


# ------------------------------------------------------------------ O1 calib stats
def calib_stats(X: np.ndarray):
    """Per input channel activation scale from calibration activations X [T x C].

    App. "Salient Weight Protection": a per-channel activation scale estimated in a
    calibration forward pass; read as the mean absolute activation (the convention
    of the activation-aware method the paper cites).  The root mean square is a
    second output: its square is the diagonal of X^T X / T.
    """
    X64 = X.astype(f64)
    T = X64.shape[0]
    s_absmean = np.abs(X64).sum(axis=0) / T
    s_rms = np.sqrt((X64 * X64).sum(axis=0) / T)
    return s_absmean.astype(f32), s_rms.astype(f32)


# -------------------------------------------------------------------- O2 features
def p99_rank(n: int) -> int:
    """1-based nearest-rank index of the 99th percentile: ceil(0.99 n), in integers."""
    return (99 * n + 99) // 100


def unit_features(W: np.ndarray, s: np.ndarray, G: int, unit_rows: int = 0) -> np.ndarray:
    """Table 1, dims 0-4 (weight statistics of the unit) and 9-11 (statistics of the
    activation scale over the unit's G input channels).  Returns [U x 8] fp64:
    mean, std, abs_mean, sparsity, outlier_frac, s_mean, s_std, s_max.
    std uses the population form (divide by n); P99 is the nearest-rank order
    statistic of |w|, so outlier_frac is an exact ratio of counts."""
    n_rb, n_chunks, R_u = unit_shape(W.shape[0], W.shape[1], G, unit_rows)
    U = n_rb * n_chunks
    feat = np.zeros((U, 8), dtype=f64)
    s64 = s.astype(f64)
    for u in range(U):
        w = unit_view(W, G, unit_rows, u).astype(f64).ravel()
        n = w.size
        aw = np.abs(w)
        mean = w.sum() / n
        std = math.sqrt(((w - mean) ** 2).sum() / n)
        abs_mean = aw.sum() / n
        sparsity = np.count_nonzero(aw < 1e-6) / n
        p99 = np.sort(aw)[p99_rank(n) - 1]
        outlier = np.count_nonzero(aw > 0.5 * p99) / n
        j = u % n_chunks
        sc = s64[j * G:(j + 1) * G]
        s_mean = sc.sum() / G
        s_std = math.sqrt(((sc - s_mean) ** 2).sum() / G)
        feat[u] = (mean, std, abs_mean, sparsity, outlier, s_mean, s_std, sc.max())
    return feat


# ------------------------------------------------------- O3 per-group quantizer fit
def group_stats(Wu: np.ndarray, keep=None):
    """Per group (row of the unit): min, max (exact) and S1 = sum |w| accumulated in
    fp64 in column order (exact for bf16 inputs; the fixed order makes it
    reproducible for any input).  With `keep` (bool [R_u x G], False = protected
    salient weight, Sec. 3.5) the statistics run over the kept weights only; a group
    with none kept has min = max = 0 and S1 = 0."""
    if keep is None:
        mn = Wu.min(axis=1).astype(f32)
        mx = Wu.max(axis=1).astype(f32)
        S1 = np.cumsum(np.abs(Wu.astype(f64)), axis=1)[:, -1]
        return mn, mx, S1
    any_kept = keep.any(axis=1)
    mn = np.where(any_kept, np.where(keep, Wu, np.inf).min(axis=1), 0.0).astype(f32)
    mx = np.where(any_kept, np.where(keep, Wu, -np.inf).max(axis=1), 0.0).astype(f32)
    S1 = np.cumsum(np.where(keep, np.abs(Wu.astype(f64)), 0.0), axis=1)[:, -1]
    return mn, mx, S1


def uniform_fit(mn: np.ndarray, mx: np.ndarray, p, bits: int):
    """[N] scale/offset of the uniform `bits`-bit quantizer at clip ratio p.
    Both ends of the range shrink toward zero by the same ratio p.  A step size
    below the smallest normal fp32 is degenerate: step 0, every code 0."""
    p = f32(p)
    qmax = f32(2 ** bits - 1)
    lo = (p * mn).astype(f32)                      # [N] one fp32 multiply
    hi = (p * mx).astype(f32)                      # [N]
    Rg = (hi - lo).astype(f32)                     # [N] one fp32 subtract
    delta = (Rg / qmax).astype(f32)                # [N] one fp32 divide
    degenerate = ~(delta >= FLT_MIN_NORMAL)
    delta = np.where(degenerate, f32(0), delta).astype(f32)
    with np.errstate(divide="ignore"):
        inv = (f32(1) / delta).astype(f32)         # [N] one fp32 divide (inf if degenerate)
    return lo, delta, inv, degenerate


def uniform_codes(Wu: np.ndarray, lo, delta, inv, degenerate, bits: int) -> np.ndarray:
    """[N] integer codes in [0, 2^bits - 1]: round-half-to-even of (w - lo) * inv."""
    qmax = 2 ** bits - 1
    with np.errstate(invalid="ignore", over="ignore"):
        u = (Wu - lo[:, None]).astype(f32)         # [N] one fp32 subtract
        t = (u * inv[:, None]).astype(f32)         # [N] one fp32 multiply
        q = np.rint(t)                             # [N] ties to even
    q = np.where(degenerate[:, None], 0.0, q)
    return np.clip(q, 0, qmax).astype(np.int64)


def uniform_dequant(codes, lo, delta) -> np.ndarray:
    """w_hat = lo + code * step, in fp64 from the stored fp32 lo and step."""
    return lo.astype(f64)[:, None] + codes.astype(f64) * delta.astype(f64)[:, None]


def absmean_scale(S1: np.ndarray, G) -> np.ndarray:
    """[N] per-group mean |w| as stored: fp32 rounding of S1 / G.  G may be a per-group
    count (kept weights of the group); a count of zero gives a scale of zero."""
    G = np.asarray(G, dtype=f64)
    with np.errstate(divide="ignore", invalid="ignore"):
        return np.where(G > 0, S1 / G, 0.0).astype(f32)


def ternary_fit(S1: np.ndarray, G):
    """[N] ternary absmean scale gamma; degenerate (all-zero-like) groups get 0."""
    gamma = absmean_scale(S1, G)
    degenerate = ~(gamma >= FLT_MIN_NORMAL)
    gamma = np.where(degenerate, f32(0), gamma).astype(f32)
    with np.errstate(divide="ignore"):
        inv = (f32(1) / gamma).astype(f32)
    return gamma, inv, degenerate


def ternary_codes(Wu: np.ndarray, inv, degenerate) -> np.ndarray:
    """[N] q in {-1, 0, +1}: round-half-to-even of w / gamma, clamped."""
    with np.errstate(invalid="ignore", over="ignore"):
        t = (Wu * inv[:, None]).astype(f32)        # [N] one fp32 multiply
        q = np.rint(t)
    q = np.where(degenerate[:, None], 0.0, q)
    return np.clip(q, -1, 1).astype(np.int64)


def binary_codes(Wu: np.ndarray) -> np.ndarray:
    """bit = 1 where w >= 0 (so -0.0 maps to +1), else 0."""
    return (Wu >= 0).astype(np.int64)


def weighted_sse(Wu64: np.ndarray, What: np.ndarray, a: np.ndarray, keep=None) -> float:
    """Activation-aware reconstruction error of one unit: sum a_c (w - w_hat)^2, over the
    kept weights when a mask is given."""
    d = Wu64 - What
    e = a[None, :] * d * d
    if keep is not None:
        e = np.where(keep, e, 0.0)
    return float(e.sum())


def fit_score_unit(Wu: np.ndarray, s_chunk: np.ndarray, clip_grid: np.ndarray, keep=None):
    """All candidate fits of one unit.  Returns (E_uniform [4 x K], E_ternary,
    E_binary, ref_energy), raw weighted sums of squares in fp64.  With `keep`, protected
    weights take no part: not in the group statistics, not in the errors."""
    Wu = np.ascontiguousarray(Wu, dtype=f32)
    R_u, G = Wu.shape
    Wu64 = Wu.astype(f64)
    a = s_chunk.astype(f64) ** 2
    mn, mx, S1 = group_stats(Wu, keep)
    n_g = G if keep is None else keep.sum(axis=1)
    K = len(clip_grid)
    E = np.zeros((4, K), dtype=f64)
    for bi, bits in enumerate(UNIFORM_BITS):
        for k in range(K):
            lo, delta, inv, deg = uniform_fit(mn, mx, clip_grid[k], bits)
            codes = uniform_codes(Wu, lo, delta, inv, deg, bits)
            E[bi, k] = weighted_sse(Wu64, uniform_dequant(codes, lo, delta), a, keep)
    gamma, ginv, gdeg = ternary_fit(S1, n_g)
    qt = ternary_codes(Wu, ginv, gdeg)
    E_t = weighted_sse(Wu64, gamma.astype(f64)[:, None] * qt, a, keep)
    alpha = absmean_scale(S1, n_g)
    qb = binary_codes(Wu)
    E_b = weighted_sse(Wu64, alpha.astype(f64)[:, None] * (2 * qb - 1), a, keep)
    ref = weighted_sse(Wu64, np.zeros_like(Wu64), a, keep)
    return E, E_t, E_b, ref


def argmin_clip(E_row: np.ndarray) -> int:
    """Clip index with the least error; exact ties go to the largest index (the
    least clipping)."""
    m = E_row.min()
    return int(np.nonzero(E_row == m)[0][-1])


def fit_score_all_bits(W: np.ndarray, s: np.ndarray, G: int, unit_rows: int,
                       clip_grid: np.ndarray, units=None, keep=None):
    """Fit and score the six candidate quantizers of every unit.

    Returns err [U x 6] fp64 (order 8, 4, 3, 2, 1.58, 1; the uniform entries at their
    best clip index), clip_idx [U x 4] uint8, ref_energy [U] fp64 and the full table
    E [U x 4 x K].  `units` restricts the work to a list of unit indices (the other
    rows stay zero).  `keep` (bool, shape of W; False = protected) masks salient weights out."""
    clip_grid = np.asarray(clip_grid, dtype=f32)
    n_rb, n_chunks, R_u = unit_shape(W.shape[0], W.shape[1], G, unit_rows)
    U = n_rb * n_chunks
    K = len(clip_grid)
    err = np.zeros((U, N_ERR), dtype=f64)
    clip_idx = np.zeros((U, 4), dtype=np.uint8)
    ref = np.zeros(U, dtype=f64)
    table = np.zeros((U, 4, K), dtype=f64)
    for u in (range(U) if units is None else units):
        j = u % n_chunks
        ku = None if keep is None else unit_view(keep, G, unit_rows, u)
        E, E_t, E_b, r = fit_score_unit(unit_view(W, G, unit_rows, u), s[j * G:(j + 1) * G], clip_grid, ku)
        table[u] = E
        for bi in range(4):
            k = argmin_clip(E[bi])
            clip_idx[u, bi] = k
            err[u, bi] = E[bi, k]
        err[u, 4] = E_t
        err[u, 5] = E_b
        ref[u] = r
    return err, clip_idx, ref, table


# ------------------------------------------------------------------ O4 apply plan
def bytes_per_group(action: int, G: int) -> int:
    """Packed bytes of one group: ceil(G*b/8) for integer b, ceil(G/5) for ternary
    (5 trits per byte), 0 for skip."""
    if action == 0:
        return 0
    if action == 5:
        return (G + 4) // 5
    bits = ACTION_CENTIBITS[action] // 100
    return (G * bits + 7) // 8


def pack_bits(codes: np.ndarray, bits: int) -> np.ndarray:
    """LSB-first bitstream of one group: code i occupies bits [i*bits, (i+1)*bits)."""
    bit_of_code = (np.asarray(codes, dtype=np.int64)[:, None] >> np.arange(bits)) & 1      # [n x bits], bit 0 first
    return np.packbits(bit_of_code.astype(np.uint8).ravel(), bitorder="little")            # zero padded to a byte


def pack_trits(trits: np.ndarray) -> np.ndarray:
    """Five trits per byte, byte = sum_j trit_j * 3^j; the tail is zero padded."""
    n = len(trits)
    nbytes = (n + 4) // 5
    padded = np.zeros(nbytes * 5, dtype=np.int64)
    padded[:n] = trits
    return (padded.reshape(nbytes, 5) @ np.array([1, 3, 9, 27, 81])).astype(np.uint8)


def unpack_bits(data: np.ndarray, bits: int, n: int) -> np.ndarray:
    """Inverse of pack_bits: code i is bits [i*bits, (i+1)*bits) of the LSB-first stream."""
    stream = np.unpackbits(np.asarray(data, dtype=np.uint8), bitorder="little")[:n * bits].reshape(n, bits)
    return (stream.astype(np.int64) << np.arange(bits)).sum(axis=1)


def unpack_trits(data: np.ndarray, n: int) -> np.ndarray:
    """Inverse of pack_trits: trit j of a byte is (byte // 3^j) % 3."""
    d = np.asarray(data, dtype=np.int64)[:, None] // np.array([1, 3, 9, 27, 81]) % 3
    return d.ravel()[:n]


def plan_layout(action: np.ndarray, R_u: int, G: int) -> np.ndarray:
    """Byte offset of every unit's packed payload, each 16-byte aligned; entry U is
    the end of the last payload rounded up to 16 (the stream length)."""
    off = np.zeros(len(action) + 1, dtype=np.int64)
    pos = 0
    for u, a in enumerate(int(x) for x in action):
        if not 0 <= a <= 6:
            raise ValueError("action out of range")
        off[u] = pos
        pos += (bytes_per_group(a, G) * R_u + 15) // 16 * 16
    off[len(action)] = pos
    return off


def quantize_unit(Wu: np.ndarray, action: int, p, keep=None):
    """Codes, stored scale and stored offset of one unit under `action` at clip p.
    Returns (stored [R_u x G] non-negative ints, scale [R_u] f32, offset [R_u] f32,
    w_hat [R_u x G] fp64).  With `keep`, the fit runs over the kept weights and the
    stored value at a protected position is the placeholder 0 (its w_hat is unused)."""
    Wu = np.ascontiguousarray(Wu, dtype=f32)
    R_u, G = Wu.shape
    mn, mx, S1 = group_stats(Wu, keep)
    n_g = G if keep is None else keep.sum(axis=1)
    zero = np.zeros(R_u, dtype=f32)
    hold = (lambda stored: stored) if keep is None else (lambda stored: np.where(keep, stored, 0))
    if action in (1, 2, 3, 4):
        bits = ACTION_CENTIBITS[action] // 100
        lo, delta, inv, deg = uniform_fit(mn, mx, p, bits)
        codes = uniform_codes(Wu, lo, delta, inv, deg, bits)
        return hold(codes), delta, lo, uniform_dequant(codes, lo, delta)
    if action == 5:
        gamma, inv, deg = ternary_fit(S1, n_g)
        q = ternary_codes(Wu, inv, deg)
        return hold(q + 1), gamma, zero, gamma.astype(f64)[:, None] * q
    if action == 6:
        alpha = absmean_scale(S1, n_g)
        bit = binary_codes(Wu)
        return hold(bit), alpha, zero, alpha.astype(f64)[:, None] * (2 * bit - 1)
    raise ValueError("skip units have no codes")


def apply_plan(W: np.ndarray, G: int, unit_rows: int, action: np.ndarray,
               clip_idx, clip_grid: np.ndarray, code_off: np.ndarray, units=None, keep=None):
    """Materialise a plan: packed code stream, per-group scale and offset.
    clip_idx None means no clipping (p = 1).  Skip units write no codes and a zero
    scale and offset.  `units` restricts the work to some units.  `keep` (bool, shape of
    W; False = protected) masks salient weights out of the fits; their code slots hold 0."""
    clip_grid = np.asarray(clip_grid, dtype=f32)
    n_rb, n_chunks, R_u = unit_shape(W.shape[0], W.shape[1], G, unit_rows)
    U = n_rb * n_chunks
    codes = np.zeros(int(code_off[U]), dtype=np.uint8)
    scale = np.zeros(U * R_u, dtype=f32)
    offset = np.zeros(U * R_u, dtype=f32)
    for u in (range(U) if units is None else units):
        a = int(action[u])
        if a == 0:
            continue
        p = f32(1)
        if a in (1, 2, 3, 4) and clip_idx is not None:
            p = clip_grid[int(clip_idx[u, a - 1])]
        ku = None if keep is None else unit_view(keep, G, unit_rows, u)
        stored, sc, of, _ = quantize_unit(unit_view(W, G, unit_rows, u), a, p, ku)
        scale[u * R_u:(u + 1) * R_u] = sc
        offset[u * R_u:(u + 1) * R_u] = of
        bpg = bytes_per_group(a, G)
        base = int(code_off[u])
        for r in range(R_u):
            row = pack_trits(stored[r]) if a == 5 else pack_bits(stored[r], ACTION_CENTIBITS[a] // 100)
            codes[base + r * bpg: base + (r + 1) * bpg] = row
    return codes, scale, offset


# ------------------------------- iterative scale refinement (App. "Per-unit Scale Optimization")
def _weighted_sums_uniform(w64, q, a, kept):
    """Column-order fp64 sums of the weighted least-squares problem  min sum a (w - lo - q step)^2:
    S0 = sum a, S1 = sum a q, S2 = sum a q^2, T0 = sum a w, T1 = sum a q w  (plain multiplies and adds)."""
    S0 = S1 = S2 = T0 = T1 = f64(0)
    for c in range(len(w64)):
        if not kept[c]:
            continue
        aq = a[c] * q[c]
        S0 = S0 + a[c]
        S1 = S1 + aq
        S2 = S2 + aq * q[c]
        T0 = T0 + a[c] * w64[c]
        T1 = T1 + aq * w64[c]
    return S0, S1, S2, T0, T1


def refine_group_uniform(w: np.ndarray, a: np.ndarray, lo, delta, bits: int, n_iter: int, kept=None):
    """The paper fits each operator's scale by a short local optimisation of the reconstruction
    loss on the unit.  Deterministic stand-in: alternate (assign codes by the normative fp32
    steps | solve the activation-weighted least-squares problem for offset and step in closed
    form), seeded from the grid fit; the loss cannot go up in either half-step.  fp64 sums in
    column order; offset and step are rounded to fp32 after every solve [N].  An iteration whose
    problem is singular (all codes equal) or whose step would fall below the smallest normal
    fp32 stops the refinement.  Returns (lo f32, step f32)."""
    w = np.asarray(w, dtype=f32)
    w64 = w.astype(f64)
    kept = np.ones(len(w), dtype=bool) if kept is None else kept
    lo, delta = f32(lo), f32(delta)
    qmax = 2 ** bits - 1
    for _ in range(n_iter):
        if not delta >= FLT_MIN_NORMAL:
            break
        inv = f32(1) / delta                                     # [N]
        q = np.clip(np.rint(((w - lo).astype(f32) * inv).astype(f32)), 0, qmax).astype(f64)   # [N]
        S0, S1, S2, T0, T1 = _weighted_sums_uniform(w64, q, a, kept)
        det = S0 * S2 - S1 * S1
        if not det > 0:
            break
        d_new = (S0 * T1 - S1 * T0) / det
        lo_new = (T0 - S1 * d_new) / S0
        d32, lo32 = f32(d_new), f32(lo_new)
        if not d32 >= FLT_MIN_NORMAL:
            break
        lo, delta = lo32, d32
    return lo, delta


def refine_group_ternary(w: np.ndarray, a: np.ndarray, gamma, n_iter: int, kept=None):
    """Same alternation for the ternary operator: q = clamp(rne(w / gamma), -1, 1), then
    gamma = sum a q w / sum a q^2.  Returns gamma f32."""
    w = np.asarray(w, dtype=f32)
    w64 = w.astype(f64)
    kept = np.ones(len(w), dtype=bool) if kept is None else kept
    gamma = f32(gamma)
    for _ in range(n_iter):
        if not gamma >= FLT_MIN_NORMAL:
            break
        inv = f32(1) / gamma
        q = np.clip(np.rint((w * inv).astype(f32)), -1, 1).astype(f64)
        N1 = D1 = f64(0)
        for c in range(len(w)):
            if kept[c]:
                aq = a[c] * q[c]
                N1 = N1 + aq * w64[c]
                D1 = D1 + aq * q[c]
        if not D1 > 0:
            break
        g = f32(N1 / D1)
        if not g >= FLT_MIN_NORMAL:
            break
        gamma = g
    return gamma


def refine_group_binary(w: np.ndarray, a: np.ndarray, alpha, kept=None):
    """The signs are fixed, so one solve is the optimum: alpha = sum a |w| / sum a."""
    w64 = np.abs(np.asarray(w, dtype=f32).astype(f64))
    kept = np.ones(len(w64), dtype=bool) if kept is None else kept
    N1 = D1 = f64(0)
    for c in range(len(w64)):
        if kept[c]:
            N1 = N1 + a[c] * w64[c]
            D1 = D1 + a[c]
    return f32(N1 / D1) if D1 > 0 else f32(alpha)


def refine_plan(W: np.ndarray, s: np.ndarray, G: int, unit_rows: int, action, clip_idx, clip_grid, code_off,
                n_iter: int, units=None, keep=None):
    """apply_plan with refined scales: every group is seeded with its grid fit (at the unit's
    clip index), refined for n_iter alternations, and quantized by the normative steps at the
    refined parameters.  Returns (codes, scale, offset, err [U] fp64: the activation-weighted
    error of the refined plan over kept weights, 0 for skip units)."""
    clip_grid = np.asarray(clip_grid, dtype=f32)
    n_rb, n_chunks, R_u = unit_shape(W.shape[0], W.shape[1], G, unit_rows)
    U = n_rb * n_chunks
    codes = np.zeros(int(code_off[U]), dtype=np.uint8)
    scale = np.zeros(U * R_u, dtype=f32)
    offset = np.zeros(U * R_u, dtype=f32)
    err = np.zeros(U, dtype=f64)
    for u in (range(U) if units is None else units):
        act = int(action[u])
        if act == 0:
            continue
        j = u % n_chunks
        Wu = np.ascontiguousarray(unit_view(W, G, unit_rows, u), dtype=f32)
        ku = None if keep is None else unit_view(keep, G, unit_rows, u)
        a = s[j * G:(j + 1) * G].astype(f64) ** 2
        mn, mx, S1 = group_stats(Wu, ku)
        n_g = G if ku is None else ku.sum(axis=1)
        bpg = bytes_per_group(act, G)
        base = int(code_off[u])
        What = np.zeros(Wu.shape, dtype=f64)
        for r in range(R_u):
            kr = None if ku is None else ku[r]
            one = slice(r, r + 1)
            if act <= 4:
                bits = ACTION_CENTIBITS[act] // 100
                p = f32(1) if clip_idx is None else clip_grid[int(clip_idx[u, act - 1])]
                lo, delta, inv, deg = uniform_fit(mn[one], mx[one], p, bits)
                lo_r, d_r = refine_group_uniform(Wu[r], a, lo[0], delta[0], bits, n_iter, kr)
                lo1, d1 = np.array([lo_r], dtype=f32), np.array([d_r], dtype=f32)
                deg1 = ~(d1 >= FLT_MIN_NORMAL)
                with np.errstate(divide="ignore"):
                    inv1 = (f32(1) / d1).astype(f32)
                stored = uniform_codes(Wu[one], lo1, d1, inv1, deg1, bits)[0]
                What[r] = lo1.astype(f64)[0] + stored.astype(f64) * d1.astype(f64)[0]
                sc_r, of_r = d1[0], lo1[0]
            elif act == 5:
                gamma, ginv, gdeg = ternary_fit(S1[one], n_g if ku is None else n_g[one])
                g_r = np.array([refine_group_ternary(Wu[r], a, gamma[0], n_iter, kr)], dtype=f32)
                deg1 = ~(g_r >= FLT_MIN_NORMAL)
                with np.errstate(divide="ignore"):
                    inv1 = (f32(1) / g_r).astype(f32)
                q = ternary_codes(Wu[one], inv1, deg1)[0]
                stored = q + 1
                What[r] = g_r.astype(f64)[0] * q
                sc_r, of_r = g_r[0], f32(0)
            else:
                alpha = absmean_scale(S1[one], n_g if ku is None else n_g[one])
                al = refine_group_binary(Wu[r], a, alpha[0], kr) if n_iter > 0 else alpha[0]
                stored = binary_codes(Wu[one])[0]
                What[r] = f64(al) * (2 * stored - 1)
                sc_r, of_r = al, f32(0)
            if kr is not None:
                stored = np.where(kr, stored, 0)
            scale[u * R_u + r] = sc_r
            offset[u * R_u + r] = of_r
            row = pack_trits(stored) if act == 5 else pack_bits(stored, ACTION_CENTIBITS[act] // 100)
            codes[base + r * bpg: base + (r + 1) * bpg] = row
        err[u] = weighted_sse(Wu.astype(f64), What, a, ku)
    return codes, scale, offset, err


# ------------------------------------------------- dequantisation of a packed plan
def unpack_group(data: np.ndarray, action: int, G: int) -> np.ndarray:
    """Stored values (codes, trits q+1, bits) of one group from its packed bytes."""
    if action == 5:
        return unpack_trits(data, G)
    return unpack_bits(data, ACTION_CENTIBITS[action] // 100, G)


def dequant_plan(W: np.ndarray, G: int, unit_rows: int, action, code_off, codes, scale, offset, keep=None):
    """Reconstruct the weights from the packed artefact alone (codes, per-group scale and
    offset): uniform w_hat = offset + code * scale, ternary scale * (trit - 1), binary
    scale * (2 bit - 1), each as ONE fp32 fused multiply-add of the stored fp32 numbers.
    Skip units keep their 16-bit weights.  Protected slots (keep False) come out as 0: their
    values live in the INT8 side stream.  Returns w_hat fp32 of W's shape."""
    n_rb, n_chunks, R_u = unit_shape(W.shape[0], W.shape[1], G, unit_rows)
    out = np.array(W, dtype=f32, copy=True)
    for u in range(n_rb * n_chunks):
        a = int(action[u])
        if a == 0:
            continue
        rb, j = divmod(u, n_chunks)
        bpg = bytes_per_group(a, G)
        base = int(code_off[u])
        for r in range(R_u):
            stored = unpack_group(codes[base + r * bpg: base + (r + 1) * bpg], a, G).astype(f64)
            sc, of = f64(scale[u * R_u + r]), f64(offset[u * R_u + r])
            if a <= 4:
                what = of + stored * sc
            elif a == 5:
                what = sc * (stored - 1.0)
            else:
                what = sc * (2.0 * stored - 1.0)
            out[rb * R_u + r, j * G:(j + 1) * G] = what.astype(f32)   # the fp64 value of a*b+c of fp32 numbers, rounded once
    if keep is not None:
        quantized = np.repeat(np.repeat((np.asarray(action).reshape(n_rb, n_chunks) != 0), R_u, axis=0), G, axis=1)
        out[quantized & ~keep] = 0.0
    return out


def dequant_error(W: np.ndarray, s: np.ndarray, G: int, unit_rows: int, action, code_off, codes, scale, offset,
                  keep=None) -> np.ndarray:
    """Activation-weighted error of a packed plan, recomputed from the artefact: per unit
    sum a_c (w - w_hat)^2 with w_hat = offset + code * scale in fp64 from the stored fp32
    numbers (the same w_hat the fit scored).  Skip units: 0.  Protected weights are left out."""
    n_rb, n_chunks, R_u = unit_shape(W.shape[0], W.shape[1], G, unit_rows)
    U = n_rb * n_chunks
    err = np.zeros(U, dtype=f64)
    for u in range(U):
        a = int(action[u])
        if a == 0:
            continue
        j = u % n_chunks
        Wu = unit_view(W, G, unit_rows, u).astype(f64)
        ku = None if keep is None else unit_view(keep, G, unit_rows, u)
        av = s[j * G:(j + 1) * G].astype(f64) ** 2
        bpg = bytes_per_group(a, G)
        base = int(code_off[u])
        What = np.zeros_like(Wu)
        for r in range(R_u):
            stored = unpack_group(codes[base + r * bpg: base + (r + 1) * bpg], a, G).astype(f64)
            sc, of = f64(scale[u * R_u + r]), f64(offset[u * R_u + r])
            What[r] = of + stored * sc if a <= 4 else (sc * (stored - 1.0) if a == 5 else sc * (2.0 * stored - 1.0))
        err[u] = weighted_sse(Wu, What, av, ku)
    return err


def dequant_gemv(W: np.ndarray, G: int, unit_rows: int, action, code_off, codes, scale, offset, x: np.ndarray,
                 rows=None, keep=None):
    """y = W_hat x from the packed artefact (the first piece of a serving path): W_hat as
    dequant_plan reconstructs it (fp32 values; skip units keep their weights; protected slots,
    keep False, count as 0), every product and the sum over the columns in fp64, columns in order.  `rows`: compute only these rows
    of y (the others come out as 0).  Returns (y [rows] fp64, scale [rows] fp64) where
    scale[r] = sum_c |w_hat[r][c] x[c]|, the natural size of the terms of y[r]."""
    What = dequant_plan(W, G, unit_rows, action, code_off, codes, scale, offset, keep=keep).astype(f64)
    xv = np.asarray(x, dtype=f32).astype(f64)
    pick = np.arange(W.shape[0]) if rows is None else np.asarray(rows, dtype=np.int64)
    y = np.zeros(W.shape[0], dtype=f64)
    mag = np.zeros(W.shape[0], dtype=f64)
    for c in range(W.shape[1]):
        term = What[pick, c] * xv[c]
        y[pick] += term
        mag[pick] += np.abs(term)
    return y, mag


# ------------------------------------------- salient-weight protection (Sec. 3.5)
def n_protected(n_unit: int, rate_ppm: int) -> int:
    """Number of protected weights of a unit of n_unit weights at a protection rate given
    in parts per million: floor(n * rate), in integers."""
    if not 0 <= rate_ppm <= 1_000_000:
        raise ValueError("rate out of range")
    return (int(n_unit) * int(rate_ppm)) // 1_000_000


def saliency(W: np.ndarray, s: np.ndarray) -> np.ndarray:
    """App. "Salient Weight Protection": saliency of a weight = its magnitude times the
    activation scale of its input channel (a magnitude too: a scale is never negative).
    [N] one fp32 multiply per weight."""
    return (np.abs(W.astype(f32)) * np.abs(s.astype(f32))[None, :]).astype(f32)


def salient_select(W: np.ndarray, s: np.ndarray, G: int, unit_rows: int, rate_ppm: int) -> np.ndarray:
    """Protected set of every unit: its n_p = floor(rate * n) most salient weights; equal
    saliencies are taken in order of the flat index inside the unit (row major).  Returns
    `keep`, bool of W's shape, False at protected weights."""
    n_rb, n_chunks, R_u = unit_shape(W.shape[0], W.shape[1], G, unit_rows)
    sal = saliency(W, s)
    keep = np.ones(W.shape, dtype=bool)
    n_p = n_protected(R_u * G, rate_ppm)
    if n_p == 0:
        return keep
    for u in range(n_rb * n_chunks):
        key = unit_view(sal, G, unit_rows, u).ravel()
        order = np.argsort(-key.astype(f64), kind="stable")      # descending saliency, ties by flat index
        ku = np.ones(R_u * G, dtype=bool)
        ku[order[:n_p]] = False
        unit_view(keep, G, unit_rows, u)[...] = ku.reshape(R_u, G)
    return keep


def pack_mask(keep: np.ndarray) -> np.ndarray:
    """Protection mask as bytes [rows x cols/8]: bit (c mod 8) of byte c div 8 of a row is
    1 where weight (row, c) is protected."""
    return np.packbits((~keep).astype(np.uint8), axis=1, bitorder="little")


def salient_encode(W: np.ndarray, s: np.ndarray, G: int, unit_rows: int, keep: np.ndarray):
    """INT8 storage of the protected weights (Sec. 3.5: "stored in INT8").  Per unit one
    symmetric scale sigma = fp32(max|w_p| / 127) [N]; code = clamp(rne(w * fp32(1/sigma)),
    -127, 127) [N]; codes of a unit in flat-index order, units back to back.  Returns
    (codes int8 [sum n_p], prot_off int64 [U+1], sigma f32 [U], err_prot fp64 [U]) with
    err_prot = sum a_c (w - code * sigma)^2 over the unit's protected weights."""
    n_rb, n_chunks, R_u = unit_shape(W.shape[0], W.shape[1], G, unit_rows)
    U = n_rb * n_chunks
    codes, off = [], np.zeros(U + 1, dtype=np.int64)
    sigma = np.zeros(U, dtype=f32)
    err = np.zeros(U, dtype=f64)
    for u in range(U):
        j = u % n_chunks
        Wu = unit_view(W, G, unit_rows, u).astype(f32)
        prot = ~unit_view(keep, G, unit_rows, u)
        wp = Wu[prot]                                            # row-major order = flat-index order
        a = np.broadcast_to((s[j * G:(j + 1) * G].astype(f64) ** 2)[None, :], Wu.shape)[prot]
        off[u + 1] = off[u] + wp.size
        if wp.size == 0:
            continue
        sg = f32(np.abs(wp).max() / f32(127))                    # [N] one fp32 divide
        if not sg >= FLT_MIN_NORMAL:
            sg = f32(0)
        with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
            inv = f32(1) / sg                                    # [N]
            t = (wp * inv).astype(f32)                           # [N]
            q = np.rint(t)
        q = np.zeros_like(wp) if sg == 0 else np.clip(q, -127, 127)
        sigma[u] = sg
        codes.append(q.astype(np.int8))
        err[u] = float((a * (wp.astype(f64) - q.astype(f64) * f64(sg)) ** 2).sum())
    allc = np.concatenate(codes) if codes else np.zeros(0, dtype=np.int8)
    return allc, off, sigma, err


# ------------------------------- heuristic sensitivity allocator and fallback (App. E, Sec. 3.5)
def unit_saliency(W: np.ndarray, s: np.ndarray, G: int, unit_rows: int = 0) -> np.ndarray:
    """App. "Comparison with Heuristic Sensitivity Allocator": a unit's saliency score is the
    mean product of activation scale and weight magnitude over the unit.  [U] fp64."""
    n_rb, n_chunks, R_u = unit_shape(W.shape[0], W.shape[1], G, unit_rows)
    prod = np.abs(W.astype(f64)) * np.abs(s.astype(f64))[None, :]
    return np.array([unit_view(prod, G, unit_rows, u).sum() / (R_u * G) for u in range(n_rb * n_chunks)], dtype=f64)


def unit_cost_centibits(a: int, n: int, n_p: int) -> int:
    """Eq. 5 for one unit, in centibits."""
    return 1600 * n if a == 0 else ACTION_CENTIBITS[a] * (n - n_p) + 800 * n_p


def heuristic_plan(sal, n_unit, n_prot, target_centibits: int, frac_1bit_ppm: int = 0, frac_ternary_ppm: int = 0):
    """The deterministic allocator the paper compares against.  Units are ranked by saliency,
    most salient first (equal scores: lower index first).  Every unit starts at 2 bits; the
    least salient floor(U * frac_1bit) units are pushed to 1 bit and the next
    floor(U * frac_ternary) to 1.58; while the plan exceeds the budget (Eq. 1 with Eq. 5),
    units are demoted one level at a time from the least salient upward (2 -> 1.58 in a first
    sweep, 1.58 -> 1 in a second); then the most salient units are promoted 2 -> 3 wherever the
    budget permits, and after that 3 -> 4 likewise.  Returns (action uint8 [U], total
    centibits, feasible)."""
    U = len(sal)
    n_prot = [0] * U if n_prot is None else [int(x) for x in n_prot]
    n_unit = [int(x) for x in n_unit]
    order = sorted(range(U), key=lambda u: (-float(sal[u]), u))
    action = [4] * U
    n1 = (U * frac_1bit_ppm) // 1_000_000
    n158 = min((U * frac_ternary_ppm) // 1_000_000, U - n1)
    for u in order[U - n1:]:
        action[u] = 6
    for u in order[U - n1 - n158:U - n1]:
        action[u] = 5
    cost = lambda u, a: unit_cost_centibits(a, n_unit[u], n_prot[u])
    B = sum(cost(u, action[u]) for u in range(U))
    budget = target_centibits * sum(n_unit)
    while B > budget:
        changed = False
        for u in reversed(order):
            if action[u] in (4, 5):
                B += cost(u, action[u] + 1) - cost(u, action[u])
                action[u] += 1
                changed = True
                if B <= budget:
                    break
        if not changed:
            break
    for frm, to in ((4, 3), (3, 2)):
        for u in order:
            if action[u] == frm and B + cost(u, to) - cost(u, frm) <= budget:
                B += cost(u, to) - cost(u, frm)
                action[u] = to
    return np.array(action, dtype=np.uint8), B, B <= budget


def fallback_promote(action, err, ref, max_rel_err: float):
    """Sec. 3.5: when the reconstruction error of the selected operator is excessive, fall back
    to a higher-precision operator.  "Excessive" is read as err / ref_energy above a caller's
    threshold (an fp32 number; the comparison err <= thr * ref is exact, in fp64); a unit climbs
    1 -> 1.58 -> 2 -> 3 -> 4 -> 8 -> skip until it passes (skip has no error).  Returns (new
    action uint8 [U], number of units changed)."""
    out = np.array(action, dtype=np.uint8).copy()
    changed = 0
    thr = float(f32(max_rel_err))
    for u in range(len(out)):
        a = int(out[u])
        a0 = a
        while a != 0 and not (float(f32(err[u][a - 1])) <= thr * float(f32(ref[u]))):
            a -= 1
        out[u] = a
        changed += a != a0
    return out, changed


# -------------------------------------------------------------- O5 effective bits
def effective_bits(action, n_unit, n_prot=None):
    """Eq. 5.  B_i = 16 n_i for skip, else b_i (n_i - n_i^p) + 8 n_i^p.  Totals in
    centibits (bits x 100) so that 1.58 stays an integer.  Returns (sum B_i in
    centibits, sum n_i); the average bit-width is sum B / (100 sum n)."""
    total_cb = 0
    total_n = 0
    for i, a in enumerate(int(x) for x in action):
        n = int(n_unit[i])
        npr = 0 if n_prot is None else int(n_prot[i])
        if not 0 <= a <= 6 or n < 0 or not 0 <= npr <= n:
            raise ValueError("bad plan entry")
        if a == 0:
            total_cb += 1600 * n
        else:
            total_cb += ACTION_CENTIBITS[a] * (n - npr) + 800 * npr
        total_n += n
    return total_cb, total_n


def budget_feasible(total_centibits: int, total_weights: int, target_centibits: int) -> bool:
    """Eq. 1 with B_target = b_target * sum n_i."""
    return total_centibits <= target_centibits * total_weights
