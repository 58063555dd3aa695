"""Pins of the oracle's salient-weight protection (Sec. 3.5 and App. "Salient Weight
Protection"; Eq. 5) against things other than itself: brute force in plain Python on tiny
inputs, constructed cases with known answers, golden bytes."""
import numpy as np
import pytest

from oracle import windq_oracle as O

f32 = np.float32


def test_n_protected_is_floor_in_integers():
    assert O.n_protected(4096 * 128, 30000) == 15728            # 3 % of 524288 = 15728.64
    assert O.n_protected(100, 30000) == 3
    assert O.n_protected(33, 30000) == 0                        # 0.99
    assert O.n_protected(34, 30000) == 1                        # 1.02
    assert O.n_protected(77, 0) == 0 and O.n_protected(77, 1_000_000) == 77
    with pytest.raises(ValueError):
        O.n_protected(10, 1_000_001)


def brute_force_protected(W, s, G, unit_rows, rate_ppm):
    """Plain Python: per unit, sort (saliency descending, flat index ascending), take n_p."""
    R, C = W.shape
    R_u = R if unit_rows == 0 else unit_rows
    prot = set()
    for rb in range(R // R_u):
        for j in range(C // G):
            items = []
            for r in range(R_u):
                for c in range(G):
                    w = f32(abs(f32(W[rb * R_u + r, j * G + c])))
                    key = f32(w * f32(abs(f32(s[j * G + c]))))
                    items.append((-float(key), r * G + c, rb * R_u + r, j * G + c))
            items.sort()
            n_p = (len(items) * rate_ppm) // 1_000_000
            prot.update((it[2], it[3]) for it in items[:n_p])
    return prot


@pytest.mark.parametrize("unit_rows,rate", [(0, 30000), (4, 125000), (0, 500000), (2, 1_000_000)])
def test_salient_select_equals_brute_force(unit_rows, rate):
    rng = np.random.default_rng(5)
    W = rng.standard_normal((8, 24)).astype(f32)
    W[rng.random(W.shape) < 0.3] = f32(0.5)                     # many equal magnitudes: ties in saliency
    s = rng.uniform(0.1, 4.0, 24).astype(f32)
    s[3] = s[4]                                                 # equal scales keep those ties alive
    keep = O.salient_select(W, s, 8, unit_rows, rate)
    prot = {(int(r), int(c)) for r, c in zip(*np.nonzero(~keep))}
    assert prot == brute_force_protected(W, s, 8, unit_rows, rate)


def test_ties_go_to_the_lowest_flat_indices():
    W = np.full((6, 16), 0.25, dtype=f32)
    s = np.ones(16, dtype=f32)
    keep = O.salient_select(W, s, 8, 3, 250000)                 # units of 3 x 8 = 24 weights, 6 protected
    for rb in range(2):
        for j in range(2):
            blk = keep[rb * 3:(rb + 1) * 3, j * 8:(j + 1) * 8]
            assert not blk[0, :6].any() and blk[0, 6:].all() and blk[1:].all()


def test_a_loud_channel_is_protected_first():
    rng = np.random.default_rng(6)
    W = (0.02 * rng.standard_normal((32, 16))).astype(f32)
    W[W == 0] = f32(0.01)
    s = np.ones(16, dtype=f32)
    s[5] = 1e6                                                  # every weight of column 5 outranks all others
    keep = O.salient_select(W, s, 16, 0, 62500)                 # 32 of 512
    assert not keep[:, 5].any() and keep[:, :5].all() and keep[:, 6:].all()
    # a negative scale counts by its magnitude
    s[5] = -1e6
    assert np.array_equal(O.salient_select(W, s, 16, 0, 62500), keep)


def test_mask_bytes_are_lsb_first_per_row():
    keep = np.ones((2, 16), dtype=bool)
    keep[0, 0] = keep[0, 9] = keep[1, 7] = keep[1, 8] = keep[1, 15] = False
    assert O.pack_mask(keep).tolist() == [[0x01, 0x02], [0x80, 0x81]]


def test_masked_fit_equals_the_fit_of_the_remaining_weights():
    """Removing the protected weight from the group is the same as masking it: statistics,
    codes of the others and every error."""
    rng = np.random.default_rng(7)
    G = 12
    Wu = (0.02 * rng.standard_normal((5, G))).astype(f32)
    Wu[:, 4] = f32(3.0)                                          # one outlier per group, all in column 4
    s = rng.uniform(0.5, 2.0, G).astype(f32)
    keep = np.ones_like(Wu, dtype=bool)
    keep[:, 4] = False
    grid = np.linspace(0.5, 1.0, 6).astype(f32)
    E, Et, Eb, ref = O.fit_score_unit(Wu, s, grid, keep)
    cols = [c for c in range(G) if c != 4]
    E2, Et2, Eb2, ref2 = O.fit_score_unit(Wu[:, cols], s[cols], grid)
    # (the two sums run over 12 and 11 columns: same terms, different fp64 summation trees)
    assert np.allclose(E, E2, rtol=1e-13, atol=0) and Et == pytest.approx(Et2, rel=1e-13)
    assert Eb == pytest.approx(Eb2, rel=1e-13) and ref == pytest.approx(ref2, rel=1e-13)
    E0 = O.fit_score_unit(Wu, s, grid)[0]
    assert np.all(E0[:, -1] > 10 * E[:, -1])                     # the outlier had been stretching every grid
    for a in range(1, 7):
        st, sc, of, _ = O.quantize_unit(Wu, a, f32(0.9), keep)
        st2, sc2, of2, _ = O.quantize_unit(Wu[:, cols], a, f32(0.9))
        assert np.array_equal(st[:, cols], st2) and np.all(st[:, 4] == 0)
        assert np.array_equal(sc, sc2) and np.array_equal(of, of2)


def test_no_protection_changes_nothing():
    rng = np.random.default_rng(8)
    W = (0.02 * rng.standard_normal((16, 32))).astype(f32)
    s = rng.uniform(0.5, 2.0, 32).astype(f32)
    grid = np.linspace(0.5, 1.0, 5).astype(f32)
    keep = O.salient_select(W, s, 16, 0, 0)
    assert keep.all()
    a = O.fit_score_all_bits(W, s, 16, 0, grid)
    b = O.fit_score_all_bits(W, s, 16, 0, grid, keep=keep)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))


def test_fully_protected_group_is_degenerate():
    Wu = np.arange(16, dtype=f32).reshape(2, 8) - 3
    keep = np.ones_like(Wu, dtype=bool)
    keep[1] = False
    mn, mx, S1 = O.group_stats(Wu, keep)
    assert mn[1] == 0 and mx[1] == 0 and S1[1] == 0 and mn[0] == -3 and mx[0] == 4
    for a in range(1, 7):
        st, sc, of, _ = O.quantize_unit(Wu, a, f32(1), keep)
        assert np.all(st[1] == 0) and sc[1] == 0 and of[1] == 0


def test_int8_codes_of_values_on_the_grid_are_exact():
    ks = np.array([127, -127, 5, 0, -64, 100, 1, -1], dtype=np.int64)
    W = np.zeros((2, 8), dtype=f32)
    W[0] = ks * 2.0 ** -10                                       # max |w| = 127 * 2^-10 -> sigma = 2^-10
    W[1] = 1e-3                                                  # kept weights
    keep = np.ones_like(W, dtype=bool)
    keep[0] = False
    s = np.linspace(1, 2, 8).astype(f32)
    codes, off, sigma, err = O.salient_encode(W, s, 8, 0, keep)
    assert off.tolist() == [0, 8] and sigma[0] == f32(2.0 ** -10)
    assert codes.tolist() == ks.tolist() and err[0] == 0.0


def test_int8_error_bound_and_order():
    rng = np.random.default_rng(9)
    W = rng.standard_normal((8, 32)).astype(f32)
    s = rng.uniform(0.5, 2.0, 32).astype(f32)
    keep = O.salient_select(W, s, 16, 4, 200000)                 # units of 64 weights, 12 protected
    codes, off, sigma, err = O.salient_encode(W, s, 16, 4, keep)
    assert np.array_equal(np.diff(off), np.full(4, 12))
    for u in range(4):
        rb, j = divmod(u, 2)
        blk = W[rb * 4:(rb + 1) * 4, j * 16:(j + 1) * 16]
        prot = ~keep[rb * 4:(rb + 1) * 4, j * 16:(j + 1) * 16]
        flat = [(r * 16 + c) for r in range(4) for c in range(16) if prot[r, c]]
        vals = np.array([blk.ravel()[i] for i in flat], dtype=np.float64)
        q = codes[off[u]:off[u + 1]].astype(np.float64)
        assert np.all(np.abs(q) <= 127) and np.abs(q).max() == 127       # the largest magnitude lands on +-127
        assert np.all(np.abs(vals - q * float(sigma[u])) <= 0.5 * float(sigma[u]) * (1 + 1e-5))
        a = np.array([float(s[j * 16 + i % 16]) ** 2 for i in flat])
        assert err[u] == pytest.approx(float((a * (vals - q * float(sigma[u])) ** 2).sum()), rel=1e-12)


def test_eq5_with_three_percent_protection():
    """Eq. 5: every unit at 2 bits with 3 % protected costs 2 (n - n_p) + 8 n_p bits."""
    n = 4096 * 128
    n_p = O.n_protected(n, 30000)
    cb, tot = O.effective_bits([4, 4, 0], [n, n, n], [n_p, n_p, n_p])
    assert cb == 2 * (200 * (n - n_p) + 800 * n_p) + 1600 * n and tot == 3 * n
    assert cb / (100 * tot) == pytest.approx((2 * (2 + 6 * n_p / n) + 16) / 3, rel=1e-12)
