"""Pins for the CPU oracle: closed forms, brute force on tiny inputs, hand examples
and golden bytes.  None of the expected values here comes from the oracle itself or
from the HIP path."""
import math
import os

import numpy as np
import pytest
from scipy import integrate, stats

from oracle import windq_oracle as O

f32 = np.float32
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------- O1 calib stats
def test_calib_constant_magnitude_gives_that_magnitude():
    sig = np.array([0.25, 1.0, 3.0, 1e-3], dtype=f32)
    sign = rng(0).choice([-1.0, 1.0], size=(64, 4)).astype(f32)
    s_abs, s_rms = O.calib_stats(sign * sig[None, :])
    assert np.array_equal(s_abs, sig)
    assert np.array_equal(s_rms, sig)


def test_calib_gaussian_ratio_and_gram_diagonal():
    T, C = 40000, 6
    sig = np.array([0.1, 0.5, 1, 2, 5, 10.0])
    X = (rng(1).standard_normal((T, C)) * sig).astype(f32)
    s_abs, s_rms = O.calib_stats(X)
    assert np.allclose(s_abs / sig, math.sqrt(2 / math.pi), atol=4 / math.sqrt(T))
    gram = X.astype(np.float64).T @ X.astype(np.float64) / T      # the dense Gram, diagonal only
    assert np.allclose(s_rms.astype(np.float64) ** 2, np.diag(gram), rtol=1e-6)


def test_calib_is_per_column_not_per_row():
    X = np.zeros((3, 2), dtype=f32)
    X[:, 0] = [1, -2, 3]
    X[:, 1] = [0, 0, -6]
    s_abs, s_rms = O.calib_stats(X)
    assert np.array_equal(s_abs, np.array([2.0, 2.0], dtype=f32))
    assert np.allclose(s_rms, [math.sqrt(14 / 3), math.sqrt(12.0)], rtol=1e-7)


# --------------------------------------------------------------------- O2 features
@pytest.mark.parametrize("n,rank", [(1, 1), (100, 99), (101, 100), (200, 198), (199, 198), (16384, 16221)])
def test_p99_rank_is_ceil(n, rank):
    assert O.p99_rank(n) == rank


def test_features_known_order_statistics():
    # |w| = 1..n with alternating signs in one unit of 10 rows x 20 columns
    n = 200
    w = np.arange(1, n + 1, dtype=f32) * np.where(np.arange(n) % 2 == 0, 1, -1).astype(f32)
    W = rng(2).permutation(w).reshape(10, 20).astype(f32)
    s = np.linspace(1, 20, 20).astype(f32)
    feat = O.unit_features(W, s, G=20, unit_rows=0)
    assert feat.shape == (1, 8)
    mean, std, am, sp, out, sm, ss, smax = feat[0]
    assert mean == pytest.approx(-0.5)                         # (1-2)+(3-4)+... = -100 over 200
    assert am == pytest.approx((n + 1) / 2)
    assert std == pytest.approx(math.sqrt((n + 1) * (2 * n + 1) / 6 - 0.25))
    assert sp == 0.0
    # P99 = 198th smallest = 198; |w| > 99 strictly -> 101 of 200
    assert out == pytest.approx(101 / 200)
    assert sm == pytest.approx(10.5) and smax == 20.0
    assert ss == pytest.approx(math.sqrt((20 ** 2 - 1) / 12))


def test_features_sparsity_threshold_and_units():
    W = np.zeros((4, 8), dtype=f32)
    W[:, :4] = 1.0
    W[0, 0] = 5e-7        # below 1e-6: sparse
    W[1, 0] = 1e-6        # fp32(1e-6) < 1e-6 as a real number
    W[2, 4] = 2e-6
    s = np.ones(8, dtype=f32)
    feat = O.unit_features(W, s, G=4, unit_rows=2)          # 2 row blocks x 2 chunks
    assert feat.shape == (4, 8)
    assert float(f32(1e-6)) < 1e-6
    assert feat[0, 3] == pytest.approx(2 / 8)               # unit (rows 0-1, chunk 0)
    assert feat[1, 3] == pytest.approx(8 / 8)               # rows 0-1, chunk 1: all zero
    assert feat[3, 3] == pytest.approx(7 / 8)               # rows 2-3, chunk 1: one 2e-6


def test_features_gaussian_asymptotics():
    n_r, G = 4096, 128
    sigma = 0.02
    W = (sigma * rng(3).standard_normal((n_r, G))).astype(f32)
    s = np.ones(G, dtype=f32)
    mean, std, am, sp, out = O.unit_features(W, s, G, 0)[0, :5]
    n = n_r * G
    assert abs(mean) < 5 * sigma / math.sqrt(n)
    assert std == pytest.approx(sigma, rel=5e-3)
    assert am / std == pytest.approx(math.sqrt(2 / math.pi), rel=5e-3)
    z = stats.norm.ppf(0.995)
    assert out == pytest.approx(2 * (1 - stats.norm.cdf(z / 2)), rel=2e-2)
    assert sp == pytest.approx(2 * stats.norm.pdf(0) * 1e-6 / sigma, abs=4 * math.sqrt(4e-5 / n))


# ------------------------------------------------------------------- O3 binary fit
def test_binary_scale_is_l2_optimal_by_brute_force():
    w = np.array([[0.75, -0.25, 0.5, -1.5, 0.0, 0.125, -0.375, 0.5]], dtype=f32)   # sum|w| = 4
    mn, mx, S1 = O.group_stats(w)
    alpha = O.absmean_scale(S1, 8)
    assert alpha[0] == f32(0.5)
    bit = O.binary_codes(w)
    sgn = 2 * bit - 1
    scan = np.linspace(0, 2, 4001)
    sse = ((w.astype(np.float64) - scan[:, None] * sgn) ** 2).sum(axis=1)
    assert scan[np.argmin(sse)] == pytest.approx(0.5, abs=1e-3)
    E, E_t, E_b, ref = O.fit_score_unit(w, np.ones(8, dtype=f32), np.array([1.0], dtype=f32))
    assert E_b == pytest.approx(ref - 8 * 0.25)                # sum w^2 - n alpha^2
    assert E_b == pytest.approx(sse.min(), rel=1e-6)


def test_binary_sign_of_zero_and_negative_zero():
    w = np.array([[0.0, -0.0, 1.0, -1.0]], dtype=f32)
    assert O.binary_codes(w).tolist() == [[1, 1, 1, 0]]


def test_binary_and_ternary_gaussian_closed_forms():
    R, G = 256, 1024        # wide groups: the per-group sample scale is close to its population value
    sigma = 0.02
    W = (sigma * rng(4).standard_normal((R, G))).astype(f32)
    E, E_t, E_b, ref = O.fit_score_unit(W, np.ones(G, dtype=f32), np.array([1.0], dtype=f32))
    n = R * G
    assert E_b / (n * sigma ** 2) == pytest.approx(1 - 2 / math.pi, rel=1e-2)
    g = math.sqrt(2 / math.pi)
    inner = integrate.quad(lambda z: z * z * stats.norm.pdf(z), -g / 2, g / 2)[0]
    outer = 2 * integrate.quad(lambda z: (z - g) ** 2 * stats.norm.pdf(z), g / 2, np.inf)[0]
    assert E_t / (n * sigma ** 2) == pytest.approx(inner + outer, rel=1e-2)
    assert inner + outer == pytest.approx(0.263382, abs=2e-4)
    mn, mx, S1 = O.group_stats(W)
    gamma, inv, deg = O.ternary_fit(S1, G)
    zero_frac = np.mean(O.ternary_codes(W, inv, deg) == 0)
    assert zero_frac == pytest.approx(2 * stats.norm.cdf(g / 2) - 1, rel=1e-2)


# ------------------------------------------------------------------ O3 ternary fit
def test_ternary_hand_example():
    c = 0.25
    w = (c * np.array([[-2, -1, 0, 1, 2]])).astype(f32)
    mn, mx, S1 = O.group_stats(w)
    gamma, inv, deg = O.ternary_fit(S1, 5)
    assert gamma[0] == pytest.approx(1.2 * c, rel=1e-7)
    assert O.ternary_codes(w, inv, deg).tolist() == [[-1, -1, 0, 1, 1]]
    E, E_t, E_b, ref = O.fit_score_unit(w, np.ones(5, dtype=f32), np.array([1.0], dtype=f32))
    assert E_t == pytest.approx(1.36 * c * c, rel=1e-6)


def test_ternary_exact_levels_have_zero_error_and_zero_group_is_degenerate():
    # |w| in {0, g}: mean|w| = g * 4/8 -> not g; use a group whose mean |w| equals its level:
    w = np.array([[0.5, -0.5, 0.5, -0.5], [0, 0, 0, 0]], dtype=f32)
    stored, scale, offset, what = O.quantize_unit(w, 5, f32(1))
    assert scale.tolist() == [0.5, 0.0]
    assert stored.tolist() == [[2, 0, 2, 0], [1, 1, 1, 1]]
    assert np.array_equal(what, w.astype(np.float64))


def test_ternary_ties_round_to_even():
    # gamma = mean|w| = 1; w/gamma = 0.5 -> 0 (even), 1.5 -> 2 -> clamp 1, -0.5 -> 0
    w = np.array([[0.5, 1.5, -0.5, 1.5]], dtype=f32)
    mn, mx, S1 = O.group_stats(w)
    gamma, inv, deg = O.ternary_fit(S1, 4)
    assert gamma[0] == 1.0
    assert O.ternary_codes(w, inv, deg).tolist() == [[0, 1, 0, 1]]


# ------------------------------------------------------------------ O3 uniform fit
def brute_force_uniform_sse(w64, lo, delta, qmax, a):
    """Least weighted squared error over ALL code assignments on the grid lo + c*delta."""
    grid = lo + delta * np.arange(qmax + 1)
    d2 = (w64[:, None] - grid[None, :]) ** 2
    return float((a * d2.min(axis=1)).sum())


@pytest.mark.parametrize("bits", [8, 4, 3, 2])
@pytest.mark.parametrize("p", [1.0, 0.8, 0.5])
def test_uniform_codes_are_nearest_grid_points(bits, p):
    G = 16
    r = rng(10 + bits)
    W = (0.02 * r.standard_normal((6, G))).astype(f32)
    s = (0.1 + r.random(G)).astype(f32)
    a = s.astype(np.float64) ** 2
    mn, mx, S1 = O.group_stats(W)
    lo, delta, inv, deg = O.uniform_fit(mn, mx, p, bits)
    codes = O.uniform_codes(W, lo, delta, inv, deg, bits)
    assert codes.min() >= 0 and codes.max() <= 2 ** bits - 1
    what = O.uniform_dequant(codes, lo, delta)
    for g in range(W.shape[0]):
        mine = float((a * (W[g].astype(np.float64) - what[g]) ** 2).sum())
        best = brute_force_uniform_sse(W[g].astype(np.float64), float(lo[g]), float(delta[g]), 2 ** bits - 1, a)
        assert best <= mine * (1 + 1e-12)
        assert mine <= best * (1 + 1e-5) + 1e-30
    # the stored range is the clipped min/max
    assert np.allclose(lo, p * mn, rtol=1e-7)
    assert np.allclose(lo + delta * (2 ** bits - 1), p * mx, rtol=1e-5, atol=1e-9)


def test_uniform_no_clip_invariants():
    W = (0.02 * rng(20).standard_normal((32, 64))).astype(f32)
    mn, mx, S1 = O.group_stats(W)
    for bits in O.UNIFORM_BITS:
        qmax = 2 ** bits - 1
        lo, delta, inv, deg = O.uniform_fit(mn, mx, 1.0, bits)
        codes = O.uniform_codes(W, lo, delta, inv, deg, bits)
        rows = np.arange(32)
        assert np.all(codes[rows, W.argmin(axis=1)] == 0)
        assert np.all(codes[rows, W.argmax(axis=1)] == qmax)
        resid = np.abs(W.astype(np.float64) - O.uniform_dequant(codes, lo, delta))
        assert np.all(resid <= 0.5 * delta.astype(np.float64)[:, None] * (1 + 1e-5))
        # quantising the reconstruction again gives the same codes
        again = O.uniform_codes(O.uniform_dequant(codes, lo, delta).astype(f32), lo, delta, inv, deg, bits)
        assert np.array_equal(again, codes)


def test_uniform_exact_grid_data_has_zero_error_and_known_codes():
    c = rng(21).integers(0, 16, size=(5, 32))
    c[:, 0] = 0
    c[:, 1] = 15
    W = ((c - 8) / 64.0).astype(f32)                 # lo = -8/64, step = 1/64, exactly representable
    stored, scale, offset, what = O.quantize_unit(W, 2, f32(1))       # action 2 = 4 bit
    assert np.array_equal(stored, c)
    assert np.all(scale == f32(1 / 64)) and np.all(offset == f32(-8 / 64))
    assert np.array_equal(what, W.astype(np.float64))
    E, E_t, E_b, ref = O.fit_score_unit(W, np.ones(32, dtype=f32), np.array([1.0], dtype=f32))
    assert E[1, 0] == 0.0 and E[0, 0] < 1e-12 * ref


def test_uniform_round_half_to_even():
    # lo = 0, hi = 3, 2 bits -> step 1; 0.5 -> 0, 1.5 -> 2, 2.5 -> 2
    W = np.array([[0.0, 3.0, 0.5, 1.5, 2.5]], dtype=f32)
    stored, scale, offset, _ = O.quantize_unit(W, 4, f32(1))
    assert scale[0] == 1.0 and offset[0] == 0.0
    assert stored.tolist() == [[0, 3, 0, 2, 2]]


def test_uniform_clipped_weights_saturate():
    W = np.array([[-1.0, 1.0, 0.2, -0.6, 0.6]], dtype=f32)
    stored, scale, offset, what = O.quantize_unit(W, 4, f32(0.5))      # range [-0.5, 0.5], step 1/3
    assert offset[0] == -0.5 and scale[0] == pytest.approx(1 / 3, rel=1e-7)
    assert stored[0, 0] == 0 and stored[0, 1] == 3 and stored[0, 3] == 0 and stored[0, 4] == 3
    assert what[0, 1] == pytest.approx(0.5, rel=1e-6)


def test_uniform_degenerate_groups():
    W = np.array([[0.25, 0.25, 0.25, 0.25], [0, 0, 0, 0]], dtype=f32)
    for action in (1, 2, 3, 4):
        stored, scale, offset, what = O.quantize_unit(W, action, f32(0.75))
        assert np.all(stored == 0) and np.all(scale == 0)
        assert offset.tolist() == [0.1875, 0.0]
    # a range so small that the step is subnormal is also degenerate
    tiny = np.array([[0.0, 1e-38, 5e-39, 2e-39]], dtype=f32)
    stored, scale, offset, _ = O.quantize_unit(tiny, 1, f32(1))
    assert np.all(stored == 0) and scale[0] == 0


def test_error_monotone_on_nested_grids_and_small_at_8_bits():
    R, G = 256, 128
    W = (0.02 * rng(22).standard_normal((R, G))).astype(f32)
    grid = np.linspace(0.5, 1.0, 6).astype(f32)
    E, E_t, E_b, ref = O.fit_score_unit(W, np.ones(G, dtype=f32), grid)
    e8, e4, e3, e2 = E
    assert np.all(e8 <= e4) and np.all(e4 <= e2)         # 3 | 15 | 255: nested grids at a fixed clip
    assert np.all(e4 <= e3) and np.all(e3 <= e2)         # statistical for 3 bits, holds by a wide margin
    # 8 bits, no clipping: uniform rounding noise step^2/12 per weight
    mn, mx, _ = O.group_stats(W)
    step2 = ((mx.astype(np.float64) - mn) / 255) ** 2
    assert e8[-1] == pytest.approx(G * step2.sum() / 12, rel=0.05)
    assert e8[-1] / ref < 1e-4
    # ternary and binary sit above 2 bits at its best clip
    assert e2.min() < E_t < E_b


def test_error_weighting_is_per_input_channel():
    R, G = 8, 16
    W = (0.02 * rng(23).standard_normal((R, G))).astype(f32)
    grid = np.array([0.7, 1.0], dtype=f32)
    ones = np.ones(G, dtype=f32)
    base = O.fit_score_unit(W, ones, grid)
    # one live channel: the error is that column's plain squared error
    s = np.zeros(G, dtype=f32)
    s[5] = 3.0
    only5 = O.fit_score_unit(W, s, grid)
    mn, mx, S1 = O.group_stats(W)
    lo, delta, inv, deg = O.uniform_fit(mn, mx, grid[0], 4)
    codes = O.uniform_codes(W, lo, delta, inv, deg, 4)
    col = W[:, 5].astype(np.float64) - (lo.astype(np.float64) + codes[:, 5] * delta.astype(np.float64))
    assert only5[0][1, 0] == pytest.approx(9.0 * (col ** 2).sum(), rel=1e-12)
    assert only5[3] == pytest.approx(9.0 * (W[:, 5].astype(np.float64) ** 2).sum(), rel=1e-12)
    # scaling s by c scales every error by c^2; the fits do not depend on s
    twice = O.fit_score_unit(W, 2 * ones, grid)
    assert np.allclose(twice[0], 4 * base[0], rtol=1e-12)
    assert twice[1] == pytest.approx(4 * base[1]) and twice[2] == pytest.approx(4 * base[2])
    # permuting the columns of W and s together changes nothing but summation order
    perm = rng(24).permutation(G)
    s2 = (0.5 + rng(25).random(G)).astype(f32)
    e_a = O.fit_score_unit(W, s2, grid)
    e_b = O.fit_score_unit(W[:, perm], s2[perm], grid)
    assert np.allclose(e_a[0], e_b[0], rtol=1e-12) and e_a[1] == pytest.approx(e_b[1], rel=1e-12)


def test_power_of_two_scaling_is_exact():
    R, G = 16, 32
    W = (0.02 * rng(26).standard_normal((R, G))).astype(f32)
    s = (0.5 + rng(27).random(G)).astype(f32)
    grid = np.array([0.6, 0.9, 1.0], dtype=f32)
    a = O.fit_score_unit(W, s, grid)
    b = O.fit_score_unit((W * f32(8)).astype(f32), s, grid)
    assert np.array_equal(b[0], 64 * a[0]) and b[1] == 64 * a[1] and b[2] == 64 * a[2]
    for action in range(1, 7):
        ca = O.quantize_unit(W, action, f32(0.9))
        cb = O.quantize_unit((W * f32(8)).astype(f32), action, f32(0.9))
        assert np.array_equal(ca[0], cb[0]) and np.array_equal(cb[1], 8 * ca[1])


def test_clip_choice_is_argmin_with_ties_to_least_clipping():
    assert O.argmin_clip(np.array([3.0, 1.0, 2.0, 1.0, 5.0])) == 3
    assert O.argmin_clip(np.array([0.0, 0.0, 0.0])) == 2
    W = (0.02 * rng(28).standard_normal((64, 128))).astype(f32)
    W[::7, 3] *= 12                                               # outliers make clipping pay at low bits
    s = np.ones(128, dtype=f32)
    grid = np.linspace(0.5, 1.0, 20).astype(f32)
    err, clip_idx, ref, table = O.fit_score_all_bits(W, s, 64, 32, grid)
    assert err.shape == (4, 6) and clip_idx.shape == (4, 4) and table.shape == (4, 4, 20)
    for u in range(4):
        for bi in range(4):
            assert err[u, bi] == table[u, bi].min()
            assert table[u, bi, clip_idx[u, bi]] == err[u, bi]
    # units are (row block, chunk): unit 1 = rows 0-31, columns 64-127 -> no outlier column
    assert clip_idx[0, 3] < 19        # 2-bit on the outlier chunk prefers clipping
    sub = O.fit_score_unit(W[32:64, 64:128], s[64:], grid)
    assert np.array_equal(sub[0], table[3])


@pytest.mark.parametrize("bits", [8, 4, 3, 2])
def test_clip_grid_against_a_dense_scan_of_clip_ratios(bits):
    """The clip search written out independently: for 2,001 clip ratios in [0.5, 1] (the 20 grid points among
    them), the unit's error with lo = p*min, step = p*(max-min)/(2^b-1) taken in fp64 and every weight sent to
    its nearest grid point by brute force.  At the shared points the oracle's table equals that scan; its
    choice is the scan's minimum restricted to the grid; and the dense scan, which contains the grid, is never
    worse than it."""
    r = rng(90 + bits)
    R, G, K = 6, 16, 20
    W = (0.02 * r.standard_normal((R, G))).astype(f32)
    W[:, 5] *= 6.0                                              # an outlier column: clipping pays at low bits
    s = (0.2 + r.random(G)).astype(f32)
    a = s.astype(np.float64) ** 2
    grid = (0.5 + 0.5 * np.arange(K) / (K - 1)).astype(f32)
    dense = np.unique(np.concatenate([np.linspace(0.5, 1.0, 2001), grid.astype(np.float64)]))
    assert len(dense) >= 2001
    qmax = 2 ** bits - 1
    W64 = W.astype(np.float64)
    mn, mx = W64.min(axis=1), W64.max(axis=1)

    def scan_error(p):
        total = 0.0
        for g in range(R):
            lo, step = p * mn[g], p * (mx[g] - mn[g]) / qmax
            total += brute_force_uniform_sse(W64[g], lo, step, qmax, a)
        return total

    E_dense = np.array([scan_error(p) for p in dense])
    E, _, _, _ = O.fit_score_unit(W, s, grid)
    bi = O.UNIFORM_BITS.index(bits)
    at_grid = np.array([E_dense[np.searchsorted(dense, float(pk))] for pk in grid])
    assert np.allclose(E[bi], at_grid, rtol=1e-7 * qmax + 1e-6, atol=0)      # fp32 scale/offset against fp64 ones (96 weights)
    k_scan = int(np.nonzero(at_grid == at_grid.min())[0][-1])
    k_orc = O.argmin_clip(E[bi])
    assert k_orc == k_scan or at_grid[k_orc] <= at_grid.min() * (1 + 1e-4)
    assert E_dense.min() <= at_grid.min() * (1 + 1e-12)
    # the grid is not a bad sample of the curve: its best point is within a few percent of the dense optimum
    assert E[bi].min() <= E_dense.min() * 1.25


# --------------------------------------------------------------- O4 packing / plan
def read_pack_golden():
    rows = []
    for line in open(os.path.join(GOLDEN, "pack_bytes.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        kind, codes, expect = [x.strip() for x in line.split("|")]
        rows.append((kind, np.array(codes.split(), dtype=np.int64), bytes.fromhex(expect.replace(" ", ""))))
    return rows


def test_pack_golden_bytes():
    rows = read_pack_golden()
    assert len(rows) >= 7
    for kind, codes, expect in rows:
        got = O.pack_trits(codes) if kind == "t" else O.pack_bits(codes, int(kind[1:]))
        assert bytes(got) == expect, (kind, codes)


@pytest.mark.parametrize("G", [64, 128, 40])
def test_pack_round_trip_and_sizes(G):
    r = rng(30 + G)
    for action, bits in ((1, 8), (2, 4), (3, 3), (4, 2), (6, 1)):
        codes = r.integers(0, 2 ** bits, size=G)
        packed = O.pack_bits(codes, bits)
        assert len(packed) == O.bytes_per_group(action, G) == math.ceil(G * bits / 8)
        assert np.array_equal(O.unpack_bits(packed, bits, G), codes)
    trits = r.integers(0, 3, size=G)
    packed = O.pack_trits(trits)
    assert len(packed) == O.bytes_per_group(5, G) == math.ceil(G / 5)
    assert np.array_equal(O.unpack_trits(packed, G), trits)
    assert O.bytes_per_group(0, G) == 0


def test_bytes_per_group_table():
    assert [O.bytes_per_group(a, 128) for a in range(7)] == [0, 128, 64, 48, 32, 26, 16]
    assert [O.bytes_per_group(a, 64) for a in range(7)] == [0, 64, 32, 24, 16, 13, 8]


def test_plan_layout_alignment_and_total():
    action = np.array([6, 0, 5, 3, 1, 0, 4], dtype=np.uint8)
    off = O.plan_layout(action, R_u=3, G=64)
    #       1b: 3*8=24->32 | skip 0 | tern 3*13=39->48 | 3b 3*24=72->80 | 8b 192 | 0 | 2b 48
    assert off.tolist() == [0, 32, 32, 80, 160, 352, 352, 400]
    assert np.all(off % 16 == 0)
    with pytest.raises(ValueError):
        O.plan_layout(np.array([7], dtype=np.uint8), 3, 64)


def test_apply_plan_stream_decodes_back_to_quantize_unit():
    R, C, G, ur = 8, 80, 40, 4
    W = (0.02 * rng(31).standard_normal((R, C))).astype(f32)
    grid = np.linspace(0.5, 1.0, 5).astype(f32)
    action = np.array([1, 5, 0, 3], dtype=np.uint8)        # 2 row blocks x 2 chunks
    clip_idx = np.array([[4, 3, 2, 1]] * 4, dtype=np.uint8)
    off = O.plan_layout(action, ur, G)
    codes, scale, offset = O.apply_plan(W, G, ur, action, clip_idx, grid, off)
    assert len(codes) == off[-1]
    # unit 3 = rows 4-7, cols 40-79, 3 bit at clip grid[2]
    stored, sc, of, _ = O.quantize_unit(W[4:8, 40:80], 3, grid[2])
    bpg = O.bytes_per_group(3, G)
    for r in range(ur):
        chunk = codes[off[3] + r * bpg: off[3] + (r + 1) * bpg]
        assert np.array_equal(O.unpack_bits(chunk, 3, G), stored[r])
    assert np.array_equal(scale[12:16], sc) and np.array_equal(offset[12:16], of)
    # unit 1 ternary: trits; unit 2 skipped: nothing written, zero scale
    stored, sc, of, _ = O.quantize_unit(W[0:4, 40:80], 5, f32(1))
    assert np.array_equal(O.unpack_trits(codes[off[1]: off[1] + 8], G), stored[0])
    assert off[3] == off[2] and np.all(scale[8:12] == 0)
    # without clip indices the fit uses p = 1
    codes1, scale1, _ = O.apply_plan(W, G, ur, action, None, grid, off)
    assert np.array_equal(scale1[0:4], O.quantize_unit(W[0:4, 0:40], 1, f32(1))[1])


# ------------------------------------------------------------- O5 effective bits
def test_effective_bits_hand_total_from_golden():
    rows, expect = [], None
    for line in open(os.path.join(GOLDEN, "effective_bits_eq5.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("="):
            expect = tuple(int(x) for x in line[1:].split())
        else:
            rows.append([int(x) for x in line.split()])
    rows = np.array(rows)
    assert O.effective_bits(rows[:, 0], rows[:, 1], rows[:, 2]) == expect == (3643260, 7000)


def test_effective_bits_uniform_plans_and_feasibility():
    n = np.array([16384, 524288, 1000])
    for a, cb in enumerate(O.ACTION_CENTIBITS):
        tot, tn = O.effective_bits([a] * 3, n)
        assert tn == n.sum() and tot == cb * n.sum()
    tot, tn = O.effective_bits([4, 4, 4], n)
    assert tot / (100 * tn) == 2.0
    assert O.budget_feasible(tot, tn, 200) and not O.budget_feasible(tot + 1, tn, 200)
    # protection moves only the protected share to 8 bits; skip ignores it
    assert O.effective_bits([6], [100], [10]) == (100 * 90 + 800 * 10, 100)
    assert O.effective_bits([0], [100], [10]) == (160000, 100)
    with pytest.raises(ValueError):
        O.effective_bits([7], [1])
    with pytest.raises(ValueError):
        O.effective_bits([1], [10], [11])
