"""Pins of the oracle's heuristic allocator and fallback (App. "Comparison with Heuristic
Sensitivity Allocator"; Sec. 3.5) by hand-worked examples and invariants."""
import numpy as np
import pytest

from oracle import windq_oracle as O

f32 = np.float32


def test_unit_saliency_is_the_mean_product():
    W = np.array([[1, -2, 3, -4], [0.5, 0.5, -1, 1]], dtype=f32)
    s = np.array([1, 2, 0.5, 0.25], dtype=f32)
    # chunks of 2 columns over both rows: (1*1 + 2*2 + .5*1 + .5*2)/4 and (3*.5 + 4*.25 + 1*.5 + 1*.25)/4
    assert O.unit_saliency(W, s, 2, 0).tolist() == [6.5 / 4, 3.25 / 4]
    assert O.unit_saliency(W, s, 2, 1).tolist() == [5 / 2, 2.5 / 2, 1.5 / 2, 0.75 / 2]
    assert O.unit_saliency(W, -s, 2, 0).tolist() == [6.5 / 4, 3.25 / 4]


def test_two_bit_default_is_kept_when_it_fits_exactly():
    sal = [3.0, 1.0, 2.0, 0.5]
    action, B, ok = O.heuristic_plan(sal, [100] * 4, None, 200)
    assert action.tolist() == [4, 4, 4, 4] and B == 4 * 200 * 100 and ok


def test_hand_worked_exchange():
    """Four equal units, target 2.0, the least salient quarter forced to 1 bit: that frees 100
    centibits per weight of one unit, which pays exactly one promotion 2 -> 3 of the most salient."""
    sal = [3.0, 1.0, 2.0, 0.5]
    action, B, ok = O.heuristic_plan(sal, [100] * 4, None, 200, frac_1bit_ppm=250000)
    assert action.tolist() == [3, 4, 4, 6] and B == (300 + 200 + 200 + 100) * 100 and ok
    # half forced to 1.58: frees 2 * 42 = 84 < 100: no promotion fits
    action, B, ok = O.heuristic_plan(sal, [100] * 4, None, 200, frac_ternary_ppm=500000)
    assert action.tolist() == [4, 5, 4, 5] and ok
    # a generous budget: everyone reaches 3 bits first (most salient first), then 4 bits while it fits
    action, B, ok = O.heuristic_plan(sal, [100] * 4, None, 350)
    assert action.tolist() == [2, 3, 2, 3] and B == (400 + 300 + 400 + 300) * 100 and ok


def test_protection_overhead_forces_demotions_from_the_least_salient():
    """3 % protected at 2 bits costs 2.18 bits: over a 2.0 budget.  Demotions 2 -> 1.58 walk up from
    the least salient unit until Eq. 1 holds."""
    n, n_p = 1000, 30
    sal = [5.0, 4.0, 3.0, 2.0, 1.0]
    action, B, ok = O.heuristic_plan(sal, [n] * 5, [n_p] * 5, 200)
    # cost at 2 bits: 200*970 + 800*30 = 218000; at 1.58: 158*970 + 24000 = 177260; budget 5 * 200000
    # k units at 1.58 cost 5*218000 - k*40740 <= 1000000  ->  k >= 2.21  ->  k = 3
    assert action.tolist() == [4, 4, 5, 5, 5] and ok
    assert B == 2 * 218000 + 3 * 177260
    cb, tot = O.effective_bits(action, [n] * 5, [n_p] * 5)
    assert cb == B


def test_infeasible_budget_ends_all_one_bit():
    action, B, ok = O.heuristic_plan([1.0, 2.0], [10, 10], None, 90)
    assert action.tolist() == [6, 6] and not ok and B == 2000


def test_ties_rank_by_index_and_plans_are_always_feasible_when_possible():
    rng = np.random.default_rng(11)
    for trial in range(20):
        U = int(rng.integers(1, 40))
        sal = rng.choice([0.5, 1.0, 2.0], U)
        n = rng.integers(1, 50, U) * 8
        n_p = (n * 3) // 100
        target = int(rng.integers(120, 420))
        action, B, ok = O.heuristic_plan(sal, n, n_p, target, int(rng.integers(0, 400000)), int(rng.integers(0, 400000)))
        cb, tot = O.effective_bits(action, n, n_p)
        assert cb == B and ok == (cb <= target * tot)
        floor_cb, _ = O.effective_bits([6] * U, n, n_p)
        assert ok == (floor_cb <= target * tot)                  # infeasible only if even all-1-bit is
        # monotone in saliency: a more salient unit never gets fewer bits than a less salient one of the same size
        bits = [O.ACTION_CENTIBITS[a] for a in action]
        for i in range(U):
            for j in range(U):
                if n[i] == n[j] and (sal[i] > sal[j] or (sal[i] == sal[j] and i < j)):
                    assert bits[i] >= bits[j] or not ok


def test_fallback_climbs_until_the_error_passes():
    err = np.array([[1e-6, 1e-4, 1e-3, 1e-2, 0.3, 0.5],
                    [1e-6, 1e-4, 1e-3, 1e-2, 0.05, 0.08],
                    [2.0, 2.0, 2.0, 2.0, 2.0, 2.0],
                    [0, 0, 0, 0, 0, 0]], dtype=f32)
    ref = np.ones(4, dtype=f32)
    out, n = O.fallback_promote([6, 6, 5, 0], err, ref, 0.1)
    assert out.tolist() == [4, 6, 0, 0] and n == 2        # unit 0: 0.5, 0.3 fail, 2-bit 1e-2 passes; unit 2: nothing passes -> skip
    out, n = O.fallback_promote([6, 5, 4, 3], err, ref, 1e-3)
    assert out.tolist() == [3, 3, 0, 3] and n == 3
    out, n = O.fallback_promote([1, 2, 3, 4], err, ref, 10.0)
    assert out.tolist() == [1, 2, 3, 4] and n == 0
