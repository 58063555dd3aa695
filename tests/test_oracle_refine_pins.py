"""Pins of the oracle's iterative scale refinement (App. "Per-unit Scale Optimization"): the
closed-form solve against a library least-squares routine, monotone loss, exact recovery of
data that lies on a grid, and reduction to the plain plan at zero iterations."""
import numpy as np
import pytest

from oracle import windq_oracle as O

f32 = np.float32


def loss_uniform(w, a, lo, d, bits):
    w = w.astype(np.float64)
    q = np.clip(np.rint(((w.astype(f32) - f32(lo)).astype(f32) * (f32(1) / f32(d))).astype(f32)), 0, 2 ** bits - 1)
    return float((a * (w - (float(lo) + q * float(d))) ** 2).sum())


def test_one_solve_is_the_weighted_least_squares_solution():
    rng = np.random.default_rng(31)
    G = 40
    w = rng.standard_normal(G).astype(f32)
    a = rng.uniform(0.1, 4.0, G)
    lo0, d0 = f32(w.min()), f32((w.max() - w.min()) / 15)
    lo1, d1 = O.refine_group_uniform(w, a, lo0, d0, 4, 1)
    q = np.clip(np.rint(((w - lo0).astype(f32) * (f32(1) / d0)).astype(f32)), 0, 15).astype(np.float64)
    A = np.stack([np.ones(G), q], axis=1) * np.sqrt(a)[:, None]
    sol = np.linalg.lstsq(A, w.astype(np.float64) * np.sqrt(a), rcond=None)[0]
    assert lo1 == f32(sol[0]) or abs(float(lo1) - sol[0]) <= 1e-6 * abs(sol[0])
    assert d1 == f32(sol[1]) or abs(float(d1) - sol[1]) <= 1e-6 * abs(sol[1])
    # ternary: gamma = sum a q w / sum a q^2
    g0 = f32(np.abs(w).mean())
    g1 = O.refine_group_ternary(w, a, g0, 1)
    qt = np.clip(np.rint((w * (f32(1) / g0)).astype(f32)), -1, 1).astype(np.float64)
    assert float(g1) == pytest.approx(float((a * qt * w).sum() / (a * qt * qt).sum()), rel=1e-6)
    # binary: the weighted mean of |w|
    assert float(O.refine_group_binary(w, a, g0)) == pytest.approx(float((a * np.abs(w)).sum() / a.sum()), rel=1e-6)


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_loss_never_goes_up_and_beats_the_grid_fit(bits):
    rng = np.random.default_rng(32)
    G = 128
    better = 0
    for trial in range(20):
        w = (0.02 * rng.standard_normal(G)).astype(f32)
        w[rng.integers(0, G, 2)] *= 6
        a = rng.uniform(0.1, 4.0, G) ** 2
        p = f32(rng.choice([0.6, 0.8, 1.0]))
        lo0 = f32(p * w.min())
        d0 = f32((f32(p * w.max()) - lo0) / f32(2 ** bits - 1))
        prev = loss_uniform(w, a, lo0, d0, bits)
        first = prev
        for it in range(1, 6):
            lo, d = O.refine_group_uniform(w, a, lo0, d0, bits, it)
            cur = loss_uniform(w, a, lo, d, bits)
            assert cur <= prev * (1 + 1e-5), (bits, trial, it)
            prev = cur
        better += prev < 0.999 * first
    assert better >= (8 if bits == 8 else 15)


def test_data_on_a_grid_is_recovered_exactly():
    rng = np.random.default_rng(33)
    q = rng.integers(0, 16, 64)
    q[0], q[1] = 0, 15
    w = (f32(-0.375) + q.astype(f32) * f32(0.0625)).astype(f32)          # exact in fp32
    a = rng.uniform(0.5, 2.0, 64)
    # a seed that is off (slightly wrong step and offset) but still assigns the right codes
    lo, d = O.refine_group_uniform(w, a, f32(-0.37), f32(0.0620), 4, 1)
    assert abs(float(lo) + 0.375) < 1e-7 and abs(float(d) - 0.0625) < 1e-8
    assert loss_uniform(w, a, lo, d, 4) < 1e-12
    # ternary data exactly on {-g, 0, g}
    wt = (f32(0.3) * rng.integers(-1, 2, 64)).astype(f32)
    wt[:3] = [f32(0.3), f32(-0.3), 0]
    g = O.refine_group_ternary(wt, a, f32(0.25), 2)
    assert g == f32(0.3)


def test_degenerate_groups_stop_cleanly():
    a = np.ones(8)
    lo, d = O.refine_group_uniform(np.full(8, 0.5, dtype=f32), a, f32(0.5), f32(0), 4, 3)
    assert lo == f32(0.5) and d == 0
    w = np.array([0.1] * 7 + [0.1000001], dtype=f32)                     # every code equal: singular, keep the seed
    lo, d = O.refine_group_uniform(w, a, f32(0.0), f32(1.0), 2, 3)
    assert lo == 0 and d == 1
    assert O.refine_group_ternary(np.zeros(8, dtype=f32), a, f32(0), 3) == 0
    assert O.refine_group_ternary(np.full(8, 1e-3, dtype=f32), a, f32(1.0), 3) == f32(1.0)    # all codes 0: no solve


def test_zero_iterations_is_the_plain_plan_and_refinement_lowers_the_unit_error():
    rng = np.random.default_rng(34)
    R, C, G = 16, 64, 32
    W = (0.02 * rng.standard_normal((R, C))).astype(f32)
    W[:, 7] *= 15
    s = rng.uniform(0.2, 3.0, C).astype(f32)
    grid = np.linspace(0.5, 1.0, 6).astype(f32)
    err, clip_idx, ref, _ = O.fit_score_all_bits(W, s, G, 0, grid)
    keep = O.salient_select(W, s, G, 0, 50000)
    for kp in (None, keep):
        e_fit = O.fit_score_all_bits(W, s, G, 0, grid, keep=kp)[0] if kp is not None else err
        ci = O.fit_score_all_bits(W, s, G, 0, grid, keep=kp)[1] if kp is not None else clip_idx
        for a_id in range(1, 7):
            action = np.full(2, a_id, dtype=np.uint8)
            off = O.plan_layout(action, R, G)
            c0, s0, o0 = O.apply_plan(W, G, 0, action, ci, grid, off, keep=kp)
            c1, s1, o1, e1 = O.refine_plan(W, s, G, 0, action, ci, grid, off, 0, keep=kp)
            assert np.array_equal(c0, c1) and np.array_equal(s0, s1) and np.array_equal(o0, o1)
            assert np.allclose(e1, e_fit[:, a_id - 1], rtol=1e-12)
            c3, s3, o3, e3 = O.refine_plan(W, s, G, 0, action, ci, grid, off, 3, keep=kp)
            assert np.all(e3 <= e_fit[:, a_id - 1] * (1 + 1e-6))
            e_back = O.dequant_error(W, s, G, 0, action, off, c3, s3, o3, keep=kp)
            assert np.allclose(e_back, e3, rtol=1e-12)
