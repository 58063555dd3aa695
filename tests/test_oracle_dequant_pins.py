"""Pins of the oracle's dequantisation of a packed plan: hand-decoded bytes, and the loop
codes -> error closing on the error the fit reported."""
import numpy as np

from oracle import windq_oracle as O

f32 = np.float32


def test_hand_decoded_groups():
    G = 8
    W = np.zeros((1, 4 * G), dtype=f32)
    W[0, 3 * G:] = np.arange(G)                               # the skip unit keeps its weights
    action = np.array([4, 5, 6, 0], dtype=np.uint8)
    off = O.plan_layout(action, 1, G)
    assert off.tolist() == [0, 16, 32, 48, 48]
    codes = np.zeros(48, dtype=np.uint8)
    codes[0:2] = [0xE4, 0x1B]                                 # 2-bit codes 0,1,2,3, 3,2,1,0
    codes[16:18] = [2 + 3 + 0 + 27 + 162, 1 + 6 + 9]          # trits 2,1,0,1,2, 1,2,1
    codes[32] = 0b00000101                                    # bits 1,0,1,0,0,0,0,0
    scale = np.array([0.5, 0.25, 2.0, 0.0], dtype=f32)
    offset = np.array([-1.0, 0.0, 0.0, 0.0], dtype=f32)
    What = O.dequant_plan(W, G, 0, action, off, codes, scale, offset)
    assert What[0, :G].tolist() == [-1, -0.5, 0, 0.5, 0.5, 0, -0.5, -1]
    assert What[0, G:2 * G].tolist() == [0.25, 0, -0.25, 0, 0.25, 0, 0.25, 0]
    assert What[0, 2 * G:3 * G].tolist() == [2, -2, 2, -2, -2, -2, -2, -2]
    assert What[0, 3 * G:].tolist() == list(range(G))
    s = np.ones(4 * G, dtype=f32)
    err = O.dequant_error(W, s, G, 0, action, off, codes, scale, offset)
    assert err.tolist() == [2 * (1 + 0.25 + 0 + 0.25), 4 * 0.0625, 8 * 4.0, 0.0]


def test_error_from_the_packed_artefact_equals_the_error_the_fit_reported():
    rng = np.random.default_rng(21)
    R, C, G = 24, 64, 16
    W = (0.02 * rng.standard_normal((R, C))).astype(f32)
    W[:, 5] *= 20
    s = rng.uniform(0.2, 3.0, C).astype(f32)
    grid = np.linspace(0.5, 1.0, 7).astype(f32)
    for unit_rows in (0, 8):
        err, clip_idx, ref, table = O.fit_score_all_bits(W, s, G, unit_rows, grid)
        U = err.shape[0]
        R_u = R if unit_rows == 0 else unit_rows
        for shift in range(7):
            action = ((np.arange(U) + shift) % 7).astype(np.uint8)
            off = O.plan_layout(action, R_u, G)
            codes, scale, offset = O.apply_plan(W, G, unit_rows, action, clip_idx, grid, off)
            e = O.dequant_error(W, s, G, unit_rows, action, off, codes, scale, offset)
            for u in range(U):
                want = 0.0 if action[u] == 0 else err[u, action[u] - 1]
                assert abs(e[u] - want) <= 1e-12 * want
            What = O.dequant_plan(W, G, unit_rows, action, off, codes, scale, offset)
            skip_cols = np.repeat(action.reshape(-1, C // G) == 0, G, axis=1)
            assert np.array_equal(What[np.repeat(skip_cols, R_u, axis=0)], W[np.repeat(skip_cols, R_u, axis=0)])


def test_protected_slots_are_left_out():
    rng = np.random.default_rng(22)
    W = (0.02 * rng.standard_normal((16, 32))).astype(f32)
    s = rng.uniform(0.2, 3.0, 32).astype(f32)
    grid = np.linspace(0.5, 1.0, 5).astype(f32)
    keep = O.salient_select(W, s, 16, 0, 100000)
    err, clip_idx, ref, _ = O.fit_score_all_bits(W, s, 16, 0, grid, keep=keep)
    action = np.array([4, 5], dtype=np.uint8)
    off = O.plan_layout(action, 16, 16)
    codes, scale, offset = O.apply_plan(W, 16, 0, action, clip_idx, grid, off, keep=keep)
    e = O.dequant_error(W, s, 16, 0, action, off, codes, scale, offset, keep=keep)
    assert abs(e[0] - err[0, 3]) <= 1e-12 * err[0, 3] and abs(e[1] - err[1, 4]) <= 1e-12 * err[1, 4]
    What = O.dequant_plan(W, 16, 0, action, off, codes, scale, offset, keep=keep)
    assert np.all(What[~keep] == 0)


def test_gemv_hand_example():
    """The packed groups of test_hand_decoded_groups, one row of four units: y = sum w_hat x by hand."""
    G = 8
    W = np.zeros((1, 4 * G), dtype=f32)
    W[0, 3 * G:] = np.arange(G)
    action = np.array([4, 5, 6, 0], dtype=np.uint8)
    off = O.plan_layout(action, 1, G)
    codes = np.zeros(48, dtype=np.uint8)
    codes[0:2] = [0xE4, 0x1B]
    codes[16:18] = [2 + 3 + 0 + 27 + 162, 1 + 6 + 9]
    codes[32] = 0b00000101
    scale = np.array([0.5, 0.25, 2.0, 0.0], dtype=f32)
    offset = np.array([-1.0, 0.0, 0.0, 0.0], dtype=f32)
    x = np.zeros(4 * G, dtype=f32)
    x[[0, 3, G, G + 2, 2 * G + 1, 2 * G + 2, 3 * G + 7]] = [2, 4, 8, -4, 0.5, 1, 3]
    # w_hat at those columns: -1, 0.5 | 0.25, -0.25 | -2, 2 | 7
    y, mag = O.dequant_gemv(W, G, 0, action, off, codes, scale, offset, x)
    assert y.tolist() == [-2 + 2 + 2 + 1 - 1 + 2 + 21]
    assert mag.tolist() == [2 + 2 + 2 + 1 + 1 + 2 + 21]


def test_gemv_picks_columns_is_linear_and_reduces_to_a_matrix_product():
    rng = np.random.default_rng(31)
    R, C, G = 12, 48, 16
    W = (0.05 * rng.standard_normal((R, C))).astype(f32)
    s = rng.uniform(0.2, 3.0, C).astype(f32)
    grid = np.linspace(0.6, 1.0, 5).astype(f32)
    err, clip_idx, ref, table = O.fit_score_all_bits(W, s, G, 4, grid)
    U = err.shape[0]
    action = (np.arange(U) % 7).astype(np.uint8)
    off = O.plan_layout(action, 4, G)
    codes, scale, offset = O.apply_plan(W, G, 4, action, clip_idx, grid, off)
    What = O.dequant_plan(W, G, 4, action, off, codes, scale, offset)
    # a unit vector picks a column of the reconstruction
    for k in (0, 17, 47):
        e = np.zeros(C, dtype=f32)
        e[k] = 1
        y, _ = O.dequant_gemv(W, G, 4, action, off, codes, scale, offset, e)
        assert np.array_equal(y, What[:, k].astype(np.float64))
    # linear in x (exactly representable combinations, so only the fp64 sums round)
    x1 = rng.integers(-8, 9, C).astype(f32)
    x2 = rng.integers(-8, 9, C).astype(f32)
    y1, _ = O.dequant_gemv(W, G, 4, action, off, codes, scale, offset, x1)
    y2, _ = O.dequant_gemv(W, G, 4, action, off, codes, scale, offset, x2)
    y12, mag = O.dequant_gemv(W, G, 4, action, off, codes, scale, offset, 2 * x1 - 3 * x2)
    assert np.all(np.abs(y12 - (2 * y1 - 3 * y2)) <= 1e-13 * (mag + 1))
    # a plan that skips every unit leaves the weights: the product with the matrix itself (BLAS, fp64)
    skip = np.zeros(U, dtype=np.uint8)
    y, mag = O.dequant_gemv(W, G, 4, skip, O.plan_layout(skip, 4, G), np.zeros(16, np.uint8), scale * 0, offset * 0, x1)
    assert np.all(np.abs(y - W.astype(np.float64) @ x1.astype(np.float64)) <= 1e-13 * mag)
    # only the requested rows
    yr, _ = O.dequant_gemv(W, G, 4, action, off, codes, scale, offset, x1, rows=[3, 9])
    assert yr[3] == y1[3] and yr[9] == y1[9] and np.count_nonzero(yr) <= 2
