"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, validates arguments before any launch, and its pure-host
entry points (plan layout, bytes per group, effective bits of Eq. 5, workspace sizes)
agree with hand-computed values and with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

from oracle import windq_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "windq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(windq_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(windq):
    names = header_functions()
    assert set(names) == set(windq.EXPORTS)
    lib = windq.lib()
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(windq):
    lib = windq.lib()
    seen = {lib.windq_status_str(i) for i in range(6)}
    assert len(seen) == 6 and lib.windq_status_str(0) == b"ok"
    assert lib.windq_status_str(99) == b"unknown status"


def test_bytes_per_group_matches_hand_table_and_oracle(windq):
    assert [windq.windq_bytes_per_group(a, 128) for a in range(7)] == [0, 128, 64, 48, 32, 26, 16]
    assert [windq.windq_bytes_per_group(a, 64) for a in range(7)] == [0, 64, 32, 24, 16, 13, 8]
    for G in (8, 40, 256, 512):
        for a in range(7):
            assert windq.windq_bytes_per_group(a, G) == O.bytes_per_group(a, G)
    assert windq.windq_bytes_per_group(7, 64) == -1 and windq.windq_bytes_per_group(1, 0) == -1


def test_plan_layout_hand_example_and_oracle(windq):
    action = torch.tensor([6, 0, 5, 3, 1, 0, 4], dtype=torch.uint8)
    off = windq.windq_plan_layout(action, 3, 64)
    assert off.tolist() == [0, 32, 32, 80, 160, 352, 352, 400]
    g = torch.Generator().manual_seed(5)
    action = torch.randint(0, 7, (1000,), generator=g, dtype=torch.uint8)
    for R_u, G in ((128, 128), (4096, 64), (7, 40)):
        off = windq.windq_plan_layout(action, R_u, G)
        assert np.array_equal(off.numpy(), O.plan_layout(action.numpy(), R_u, G))
        assert torch.all(off % 16 == 0)
    with pytest.raises(windq.WindqError) as e:
        windq.windq_plan_layout(torch.tensor([1, 7], dtype=torch.uint8), 4, 64)
    assert e.value.status == windq.WINDQ_EINVAL
    assert windq.windq_plan_layout(torch.zeros(0, dtype=torch.uint8), 4, 64).tolist() == [0]


def test_effective_bits_hand_totals(windq):
    # Eq. 5 hand example: one unit per action, n = 1000, 30 protected -> 36432.6 bits
    action = torch.arange(7, dtype=torch.uint8)
    n = torch.full((7,), 1000, dtype=torch.int64)
    npr = torch.full((7,), 30, dtype=torch.int64)
    assert windq.windq_effective_bits(action, n, npr) == (3643260, 7000)
    assert windq.windq_effective_bits(action, n) == ((1600 + 800 + 400 + 300 + 200 + 158 + 100) * 1000, 7000)
    two = torch.full((5,), 4, dtype=torch.uint8)
    n5 = torch.tensor([16384, 524288, 1, 7, 100000], dtype=torch.int64)
    cb, nw = windq.windq_effective_bits(two, n5)
    assert cb == 200 * nw and nw == int(n5.sum())
    g = torch.Generator().manual_seed(6)
    a = torch.randint(0, 7, (5000,), generator=g, dtype=torch.uint8)
    nn = torch.randint(1, 1 << 20, (5000,), generator=g, dtype=torch.int64)
    pp = (nn.double() * 0.03).long()
    assert windq.windq_effective_bits(a, nn, pp) == O.effective_bits(a.numpy(), nn.numpy(), pp.numpy())
    for bad in ((torch.tensor([7], dtype=torch.uint8), torch.tensor([1]), None),
                (torch.tensor([1], dtype=torch.uint8), torch.tensor([-1]), None),
                (torch.tensor([1], dtype=torch.uint8), torch.tensor([5]), torch.tensor([6]))):
        with pytest.raises(windq.WindqError) as e:
            windq.windq_effective_bits(*bad)
        assert e.value.status == windq.WINDQ_EINVAL


def test_workspace_sizes(windq):
    B, F = windq.WINDQ_BF16, windq.WINDQ_F32
    # fit-score: one fp64 per (64-row tile, candidate): 32 units x 64 tiles x (4*20 errors + 3 per column quarter
    # + 20 noise terms), then a counter (256 bytes), a list of unit indices (4 bytes each, rounded up to 256) and
    # per chunk of columns 128 + 64 + 4 words of column selection
    colsel = 32 * (128 + 64 + 4) * 4
    assert colsel % 256 == 0
    assert windq.workspace_bytes(windq.CALL_FIT_SCORE, B, 4096, 4096, 128, 0, 20) == 32 * 64 * 112 * 8 + 256 + 256 + colsel
    assert windq.workspace_bytes(windq.CALL_FIT_SCORE, B, 4096, 4096, 128, 128, 20) == 1024 * 2 * 112 * 8 + 256 + 4096 + colsel
    # calib: two fp64 per (32-token slab, channel)
    assert windq.workspace_bytes(windq.CALL_CALIB_STATS, F, 256, 512) == 8 * 512 * 16
    assert windq.workspace_bytes(windq.CALL_UNIT_FEATURES, B, 4096, 4096, 128, 0, 1) > 32 * 2048 * 4
    assert windq.workspace_bytes(windq.CALL_APPLY_PLAN, B, 4096, 4096, 128, 0, 1) == 256
    # invalid shapes give 0
    assert windq.workspace_bytes(windq.CALL_FIT_SCORE, B, 4096, 4100, 128, 0, 20) == 0
    assert windq.workspace_bytes(windq.CALL_FIT_SCORE, B, 4096, 4096, 128, 100, 20) == 0
    assert windq.workspace_bytes(windq.CALL_FIT_SCORE, B, 4096, 4096, 128, 0, 65) == 0
    assert windq.workspace_bytes(windq.CALL_FIT_SCORE, 2, 4096, 4096, 128, 0, 20) == 0


def _mat(windq, rows=128, cols=128, dtype=None, data=4096, ld=None):
    return windq.windq_mat(data, windq.WINDQ_BF16 if dtype is None else dtype, 0, rows, cols, cols if ld is None else ld)


def test_argument_validation_happens_before_any_launch(windq):
    """Every error path returns before touching the GPU, so fake (never dereferenced)
    device addresses are enough and this runs without one."""
    lib = windq.lib()
    P = 4096            # a 'device pointer' that is never dereferenced on these paths
    grid = torch.linspace(0.5, 1.0, 20, dtype=torch.float32)
    gp = grid.data_ptr()
    br = ctypes.byref

    def fit(m, s=P, G=64, ur=0, g=gp, K=20, err=P, ci=P, ws=P, wsb=1 << 30):
        return lib.windq_fit_score_all_bits(br(m), s, G, ur, g, K, err, ci, None, ws, wsb, None)

    assert fit(_mat(windq, data=None)) == windq.WINDQ_EINVAL
    assert fit(_mat(windq, data=4100)) == windq.WINDQ_EINVAL            # misaligned
    assert fit(_mat(windq, dtype=5)) == windq.WINDQ_EDTYPE
    assert fit(_mat(windq, cols=100, ld=104)) == windq.WINDQ_ESHAPE      # cols % 8
    assert fit(_mat(windq, cols=192), G=128) == windq.WINDQ_ESHAPE       # cols % chunk_w
    assert fit(_mat(windq), G=12) == windq.WINDQ_ESHAPE                  # chunk_w % 8
    assert fit(_mat(windq, cols=1024), G=1024) == windq.WINDQ_ESHAPE     # chunk too wide
    assert fit(_mat(windq), ur=48) == windq.WINDQ_ESHAPE                 # unit_rows does not divide rows
    assert fit(_mat(windq, ld=120)) == windq.WINDQ_ESHAPE                # ld < cols
    assert fit(_mat(windq), s=None) == windq.WINDQ_EINVAL
    assert fit(_mat(windq), err=None) == windq.WINDQ_EINVAL
    assert fit(_mat(windq), g=None) == windq.WINDQ_EINVAL
    assert fit(_mat(windq), K=0) == windq.WINDQ_EINVAL
    assert fit(_mat(windq), K=65) == windq.WINDQ_EINVAL
    assert fit(_mat(windq), ws=None) == windq.WINDQ_EWORKSPACE
    assert fit(_mat(windq), wsb=8) == windq.WINDQ_EWORKSPACE
    bad = torch.tensor([0.5, 0.4, 1.0], dtype=torch.float32)             # not ascending
    assert fit(_mat(windq), g=bad.data_ptr(), K=3) == windq.WINDQ_EINVAL
    bad = torch.tensor([0.5, 1.5], dtype=torch.float32)                  # above 1
    assert fit(_mat(windq), g=bad.data_ptr(), K=2) == windq.WINDQ_EINVAL

    m = _mat(windq)
    assert lib.windq_calib_stats(br(m), None, None, P, 1 << 30, None) == windq.WINDQ_EINVAL
    assert lib.windq_calib_stats(br(m), P, None, None, 0, None) == windq.WINDQ_EWORKSPACE
    assert lib.windq_calib_stats(None, P, None, P, 1 << 30, None) == windq.WINDQ_EINVAL
    assert lib.windq_unit_features(br(m), None, 64, 0, P, P, 1 << 30, None) == windq.WINDQ_EINVAL
    assert lib.windq_unit_features(br(m), P, 64, 0, P, P, 16, None) == windq.WINDQ_EWORKSPACE
    assert lib.windq_unit_features(br(m), P, 60, 0, P, P, 1 << 30, None) == windq.WINDQ_ESHAPE

    def apply(action=P, ci=P, g=gp, K=20, off=P, codes=P, nbytes=1 << 20, scale=P, offset=P, ws=P):
        return lib.windq_apply_plan(br(m), 64, 0, action, ci, g, K, off, codes, nbytes, scale, offset, ws, 256, None)

    assert apply(action=None) == windq.WINDQ_EINVAL
    assert apply(off=None) == windq.WINDQ_EINVAL
    assert apply(scale=None) == windq.WINDQ_EINVAL
    assert apply(codes=None) == windq.WINDQ_EINVAL
    assert apply(codes=4100) == windq.WINDQ_EINVAL
    assert apply(g=None) == windq.WINDQ_EINVAL               # clip indices without a grid
    assert apply(ws=None) == windq.WINDQ_EWORKSPACE


def test_binding_refuses_cpu_tensors(windq):
    W = torch.zeros(64, 64, dtype=torch.bfloat16)
    s = torch.ones(64)
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        windq.windq_fit_score_all_bits(W, s, 64, 0, torch.ones(1))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        windq.windq_calib_stats(W)


# ------------------------------------------- heuristic allocator and fallback (host only)
def test_heuristic_plan_matches_hand_examples_and_oracle(windq):
    sal = torch.tensor([3.0, 1.0, 2.0, 0.5])
    n = torch.full((4,), 100, dtype=torch.int64)
    action, B, ok = windq.windq_heuristic_plan(sal, n, None, 200, frac_1bit_ppm=250000)
    assert action.tolist() == [3, 4, 4, 6] and B == 80000 and ok
    action, B, ok = windq.windq_heuristic_plan(torch.tensor([1.0, 2.0]), torch.tensor([10, 10]), None, 90)
    assert action.tolist() == [6, 6] and not ok and B == 2000
    rng = np.random.default_rng(12)
    for trial in range(50):
        U = int(rng.integers(1, 300))
        sal = torch.from_numpy(rng.choice([0.25, 0.5, 1.0, 2.0, 7.0], U).astype(np.float32) * (1 + (trial % 2) * rng.random(U).astype(np.float32)))
        n = torch.from_numpy(rng.integers(1, 50, U) * 8)
        n_p = (n * 3) // 100 if trial % 3 else None
        target = int(rng.integers(100, 450))
        f1, f158 = int(rng.integers(0, 500000)), int(rng.integers(0, 500000))
        action, B, ok = windq.windq_heuristic_plan(sal, n, n_p, target, f1, f158)
        o_action, o_B, o_ok = O.heuristic_plan(sal.numpy(), n.numpy(), None if n_p is None else n_p.numpy(), target, f1, f158)
        assert np.array_equal(action.numpy(), o_action) and B == o_B and ok == o_ok
        cb, tot = windq.windq_effective_bits(action, n, n_p)
        assert cb == B
    with pytest.raises(windq.WindqError):
        windq.windq_heuristic_plan(torch.tensor([float("nan")]), torch.tensor([8]), None, 200)
    with pytest.raises(windq.WindqError):
        windq.windq_heuristic_plan(torch.tensor([1.0]), torch.tensor([8]), torch.tensor([9]), 200)
    action, B, ok = windq.windq_heuristic_plan(torch.empty(0), torch.empty(0, dtype=torch.int64), None, 200)
    assert action.numel() == 0 and B == 0 and ok


def test_fallback_promote_matches_hand_example_and_oracle(windq):
    err = torch.tensor([[1e-6, 1e-4, 1e-3, 1e-2, 0.3, 0.5],
                        [1e-6, 1e-4, 1e-3, 1e-2, 0.05, 0.08],
                        [2.0, 2.0, 2.0, 2.0, 2.0, 2.0],
                        [0, 0, 0, 0, 0, 0]], dtype=torch.float32)
    ref = torch.ones(4)
    action = torch.tensor([6, 6, 5, 0], dtype=torch.uint8)
    assert windq.windq_fallback_promote(action, err, ref, 0.1) == 2 and action.tolist() == [4, 6, 0, 0]
    action = torch.tensor([6, 5, 4, 3], dtype=torch.uint8)
    assert windq.windq_fallback_promote(action, err, ref, 1e-3) == 3 and action.tolist() == [3, 3, 0, 3]
    rng = np.random.default_rng(13)
    for trial in range(20):
        U = int(rng.integers(1, 200))
        e = np.sort(rng.random((U, 6)).astype(np.float32) ** 4, axis=1)          # fewer bits, larger error
        r = (rng.random(U).astype(np.float32) + 0.5)
        a0 = rng.integers(0, 7, U).astype(np.uint8)
        thr = float(rng.choice([1e-3, 1e-2, 0.1, 0.5]))
        want, n_want = O.fallback_promote(a0, e, r, thr)
        a = torch.from_numpy(a0.copy())
        n_got = windq.windq_fallback_promote(a, torch.from_numpy(e), torch.from_numpy(r), thr)
        assert np.array_equal(a.numpy(), want) and n_got == n_want
    with pytest.raises(windq.WindqError):
        windq.windq_fallback_promote(torch.tensor([7], dtype=torch.uint8), err[:1], ref[:1], 0.1)


def test_argument_validation_of_the_protection_refinement_and_dequant_calls(windq):
    """Same rule for the later entry points: every error is returned before any launch."""
    lib = windq.lib()
    P, br = 4096, ctypes.byref
    grid = torch.linspace(0.5, 1.0, 20, dtype=torch.float32)
    gp = grid.data_ptr()
    m = _mat(windq)
    big = 1 << 30
    E, S, WS = windq.WINDQ_EINVAL, windq.WINDQ_ESHAPE, windq.WINDQ_EWORKSPACE
    assert windq.windq_n_protected(524288, 30000) == 15728 and windq.windq_n_protected(100, 1000001) == -1
    assert windq.windq_n_protected(-1, 10) == -1

    sel = lambda mat=m, s=P, G=64, ppm=30000, mask=P, ws=P, wsb=big: lib.windq_salient_select(br(mat), s, G, 0, ppm, mask, ws, wsb, None)
    assert sel(s=None) == E and sel(mask=None) == E and sel(ppm=1000001) == E
    assert sel(G=12) == S and sel(ws=None) == WS and sel(wsb=64) == WS
    assert sel(mat=_mat(windq, data=None)) == E

    enc = lambda codes=P, scale=P, err=P, mask=P, wsb=big: lib.windq_salient_encode(br(m), P, 64, 0, mask, 30000, codes, scale, err, P, wsb, None)
    assert enc(codes=None) == E and enc(scale=None) == E and enc(err=None) == E and enc(mask=None) == E and enc(wsb=8) == WS

    fitp = lambda mask=P, K=20: lib.windq_fit_score_all_bits_prot(br(m), P, 64, 0, mask, gp, K, P, P, None, P, big, None)
    assert fitp(mask=None) == E and fitp(K=0) == E

    appp = lambda mask=P, action=P, codes=P: lib.windq_apply_plan_prot(br(m), 64, 0, mask, action, None, None, 0, P, codes, 1 << 20, P, P, P, big, None)
    assert appp(mask=None) == E and appp(action=None) == E and appp(codes=4100) == E

    sal = lambda out=P, wsb=big: lib.windq_unit_saliency(br(m), P, 64, 0, out, P, wsb, None)
    assert sal(out=None) == E and sal(wsb=8) == WS

    deq = lambda err=P, what=None, scale=P, codes=P: lib.windq_dequant_plan(br(m), P, 64, 0, None, P, P, codes, 1 << 20, scale, P, err, what, P, big, None)
    assert deq(err=None, what=None) == E and deq(scale=None) == E and deq(codes=None) == E
    assert deq(err=None, what=4098) == E                                 # misaligned reconstruction buffer

    ref = lambda n_iter=3, err=P, K=20, g=gp, ci=P: lib.windq_refine_plan(br(m), P, 64, 0, None, P, ci, g, K, n_iter, P, P, 1 << 20, P, P, err, P, big, None)
    assert ref(n_iter=-1) == E and ref(n_iter=65) == E and ref(err=None) == E and ref(K=65) == E
    bad = torch.tensor([0.9, 0.8], dtype=torch.float32)
    assert ref(g=bad.data_ptr(), K=2) == E


def test_workspace_sizes_of_the_later_calls(windq):
    B = windq.WINDQ_BF16
    tiles = 32 * 64
    assert windq.workspace_bytes(windq.CALL_UNIT_SALIENCY, B, 4096, 4096, 128, 0, 1) == tiles * 8
    assert windq.workspace_bytes(windq.CALL_DEQUANT, B, 4096, 4096, 128, 0, 1) == tiles * 4 * 8      # 4 row passes per tile
    assert windq.workspace_bytes(windq.CALL_DEQUANT, B, 4096, 4096, 16, 0, 1) == 256 * 64 * 8
    assert windq.workspace_bytes(windq.CALL_REFINE, B, 4096, 4096, 128, 0, 1) == tiles * 8
    sal = windq.workspace_bytes(windq.CALL_SALIENT, B, 4096, 4096, 128, 0, 1)
    assert sal >= 3 * 32 * 2048 * 4 + 32 * 4096 * 4 and sal % 256 == 0
    assert windq.workspace_bytes(windq.CALL_SALIENT, B, 4096, 4100, 128, 0, 1) == 0


def test_argument_validation_of_the_batch_calls(windq):
    """The batch calls check every item before the first launch, like the per-matrix calls."""
    from paper_2605_26660_amd import binding as B
    lib = windq.lib()
    P = 4096
    grid = torch.linspace(0.5, 1.0, 20, dtype=torch.float32)
    gp = grid.data_ptr()
    good = _mat(windq)
    odd = _mat(windq, dtype=windq.WINDQ_F32)

    def fit_items(mats, ws=P, wsb=1 << 30, err=P):
        items = (B.windq_fit_item * len(mats))()
        for i, m in enumerate(mats):
            items[i] = B.windq_fit_item(ctypes.pointer(m), P, None, err, P, None, ws, wsb)
        return items

    assert lib.windq_fit_score_all_bits_batch(None, 1, 64, 0, gp, 20, None) == windq.WINDQ_EINVAL
    assert lib.windq_fit_score_all_bits_batch(fit_items([good]), 0, 64, 0, gp, 20, None) == windq.WINDQ_EINVAL
    assert lib.windq_fit_score_all_bits_batch(fit_items([good] * 9), 9, 64, 0, gp, 20, None) == windq.WINDQ_EINVAL
    assert lib.windq_fit_score_all_bits_batch(fit_items([good, odd]), 2, 64, 0, gp, 20, None) == windq.WINDQ_EINVAL
    assert lib.windq_fit_score_all_bits_batch(fit_items([good, good], err=None), 2, 64, 0, gp, 20, None) == windq.WINDQ_EINVAL
    assert lib.windq_fit_score_all_bits_batch(fit_items([good, good], wsb=8), 2, 64, 0, gp, 20, None) == windq.WINDQ_EWORKSPACE
    assert lib.windq_fit_score_all_bits_batch(fit_items([good, good]), 2, 60, 0, gp, 20, None) == windq.WINDQ_ESHAPE
    assert lib.windq_fit_score_all_bits_batch(fit_items([good, good]), 2, 64, 0, gp, 0, None) == windq.WINDQ_EINVAL

    feat = (B.windq_feat_item * 2)()
    for i in range(2):
        feat[i] = B.windq_feat_item(ctypes.pointer(good), P, P, P, 1 << 30)
    assert lib.windq_unit_features_batch(None, 1, 64, 0, None) == windq.WINDQ_EINVAL
    assert lib.windq_unit_features_batch(feat, 9, 64, 0, None) == windq.WINDQ_EINVAL
    feat[1] = B.windq_feat_item(ctypes.pointer(good), P, None, P, 1 << 30)
    assert lib.windq_unit_features_batch(feat, 2, 64, 0, None) == windq.WINDQ_EINVAL
    feat[1] = B.windq_feat_item(ctypes.pointer(good), P, P, P, 16)
    assert lib.windq_unit_features_batch(feat, 2, 64, 0, None) == windq.WINDQ_EWORKSPACE

    app = (B.windq_apply_item * 2)()
    for i in range(2):
        app[i] = B.windq_apply_item(ctypes.pointer(good), None, P, P, P, P, 1 << 20, P, P, P, 256)
    assert lib.windq_apply_plan_batch(None, 1, 64, 0, gp, 20, None) == windq.WINDQ_EINVAL
    assert lib.windq_apply_plan_batch(app, 0, 64, 0, gp, 20, None) == windq.WINDQ_EINVAL
    assert lib.windq_apply_plan_batch(app, 2, 64, 0, None, 0, None) == windq.WINDQ_EINVAL      # clip indices without a grid
    app[1] = B.windq_apply_item(ctypes.pointer(good), None, None, P, P, P, 1 << 20, P, P, P, 256)
    assert lib.windq_apply_plan_batch(app, 2, 64, 0, gp, 20, None) == windq.WINDQ_EINVAL
    app[1] = B.windq_apply_item(ctypes.pointer(good), None, P, P, P, P, 1 << 20, P, P, None, 0)
    assert lib.windq_apply_plan_batch(app, 2, 64, 0, gp, 20, None) == windq.WINDQ_EWORKSPACE

    cal = (B.windq_calib_item * 2)()
    for i in range(2):
        cal[i] = B.windq_calib_item(ctypes.pointer(good), P, None, P, 1 << 30)
    assert lib.windq_calib_stats_batch(None, 1, None) == windq.WINDQ_EINVAL
    assert lib.windq_calib_stats_batch(cal, 9, None) == windq.WINDQ_EINVAL
    cal[1] = B.windq_calib_item(ctypes.pointer(good), None, None, P, 1 << 30)
    assert lib.windq_calib_stats_batch(cal, 2, None) == windq.WINDQ_EINVAL
    cal[1] = B.windq_calib_item(ctypes.pointer(odd), P, None, P, 1 << 30)
    assert lib.windq_calib_stats_batch(cal, 2, None) == windq.WINDQ_EINVAL
    cal[1] = B.windq_calib_item(None, P, None, P, 1 << 30)
    assert lib.windq_calib_stats_batch(cal, 2, None) == windq.WINDQ_EINVAL
