"""The *_batch entry points: one launch over several matrices must give, bit for bit, what
the per-matrix calls give (each of which is checked against the oracle elsewhere)."""
import ctypes

import pytest
import torch

from paper_2605_26660_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def same_bits(a, b):
    return torch.equal(a.contiguous().view(torch.uint8).flatten(), b.contiguous().view(torch.uint8).flatten())


def block(dtype, shapes, seed):
    Ws = [synth.weights_llm(r, c, seed=seed + i, device=DEV, dtype=dtype) for i, (r, c) in enumerate(shapes)]
    gen = torch.Generator().manual_seed(seed)
    ss = [(torch.exp(torch.randn(c, generator=gen)) + 0.05).to(DEV) for _, c in shapes]
    return Ws, ss


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("G,unit_rows,K,shapes", [
    (128, 0, 20, [(256, 512), (1024, 256), (64, 128), (200, 384), (2048, 128), (192, 640), (512, 512)]),
    (64, 64, 7, [(128, 256), (64, 64), (320, 192)]),
    (8, 0, 3, [(16, 24), (8, 8)]),
    (128, 0, 40, [(300, 256)]),
])
def test_fit_score_batch_equals_single_calls(windq, dtype, G, unit_rows, K, shapes):
    Ws, ss = block(dtype, shapes, 131)
    cg = synth.clip_grid(K)
    singles = [windq.windq_fit_score_all_bits(W, s, G, unit_rows, cg) for W, s in zip(Ws, ss)]
    batch = windq.windq_fit_score_all_bits_batch(Ws, ss, G, unit_rows, cg)
    torch.cuda.synchronize()
    for one, got in zip(singles, batch):
        for a, b in zip(one, got):
            assert same_bits(a, b)


def test_fit_score_batch_rejects_bad_batches(windq):
    Ws, ss = block(torch.bfloat16, [(64, 128)] * 9, 7)
    cg = synth.clip_grid(4)
    with pytest.raises(windq.WindqError) as e:
        windq.windq_fit_score_all_bits_batch(Ws, ss, 128, 0, cg)                 # more than MAX_BATCH
    assert e.value.status == windq.WINDQ_EINVAL
    with pytest.raises(windq.WindqError) as e:
        windq.windq_fit_score_all_bits_batch([], [], 128, 0, cg)
    assert e.value.status == windq.WINDQ_EINVAL
    mixed = [Ws[0], Ws[1].float()]
    with pytest.raises(windq.WindqError) as e:
        windq.windq_fit_score_all_bits_batch(mixed, ss[:2], 128, 0, cg)           # one element type per launch
    assert e.value.status == windq.WINDQ_EINVAL
    with pytest.raises(windq.WindqError) as e:
        windq.windq_fit_score_all_bits_batch(Ws[:2], ss[:2], 96, 0, cg)           # 128 columns are not chunks of 96
    assert e.value.status == windq.WINDQ_ESHAPE
    small_ws = [torch.empty(64, dtype=torch.uint8, device=DEV)] * 2
    with pytest.raises(windq.WindqError) as e:
        windq.windq_fit_score_all_bits_batch(Ws[:2], ss[:2], 128, 0, cg, wss=small_ws)
    assert e.value.status == windq.WINDQ_EWORKSPACE


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("G,unit_rows,shapes", [
    (128, 0, [(256, 512), (1024, 256), (64, 128), (200, 384), (2048, 128), (192, 640), (512, 512)]),
    (64, 64, [(128, 256), (64, 64), (320, 192)]),
    (8, 0, [(16, 24), (8, 8)]),
    (256, 100, [(300, 256)]),
])
def test_unit_features_batch_equals_single_calls(windq, dtype, G, unit_rows, shapes):
    Ws, ss = block(dtype, shapes, 151)
    singles = [windq.windq_unit_features(W, s, G, unit_rows) for W, s in zip(Ws, ss)]
    batch = windq.windq_unit_features_batch(Ws, ss, G, unit_rows)
    torch.cuda.synchronize()
    for one, got in zip(singles, batch):
        assert same_bits(one, got)


def test_unit_features_batch_rejects_bad_batches(windq):
    Ws, ss = block(torch.bfloat16, [(64, 128)] * 9, 9)
    for bad in (lambda: windq.windq_unit_features_batch(Ws, ss, 128, 0),
                lambda: windq.windq_unit_features_batch([], [], 128, 0),
                lambda: windq.windq_unit_features_batch([Ws[0], Ws[1].float()], ss[:2], 128, 0)):
        with pytest.raises(windq.WindqError) as e:
            bad()
        assert e.value.status == windq.WINDQ_EINVAL
    with pytest.raises(windq.WindqError) as e:
        windq.windq_unit_features_batch(Ws[:2], ss[:2], 128, 0, wss=[torch.empty(64, dtype=torch.uint8, device=DEV)] * 2)
    assert e.value.status == windq.WINDQ_EWORKSPACE


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("G,unit_rows,shapes", [
    (128, 0, [(256, 512), (1024, 256), (64, 128), (200, 384), (2048, 128), (192, 640), (512, 512)]),
    (64, 64, [(128, 256), (64, 64), (320, 192)]),
    (32, 0, [(100, 96), (64, 32)]),
    (40, 0, [(70, 120), (16, 40)]),
])
def test_apply_plan_batch_equals_single_calls(windq, dtype, G, unit_rows, shapes):
    Ws, ss = block(dtype, shapes, 171)
    K = 7
    cg = synth.clip_grid(K)
    actions, idxs, offs, singles, codes_b, outs_b = [], [], [], [], [], []
    for i, (W, s) in enumerate(zip(Ws, ss)):
        U, R_u = windq.n_units(W.shape[0], W.shape[1], G, unit_rows)
        _, clip_idx, _ = windq.windq_fit_score_all_bits(W, s, G, unit_rows, cg)
        action = ((torch.arange(U) + i) % 7).to(torch.uint8)
        off = windq.windq_plan_layout(action, R_u, G)
        actions.append(action.to(DEV)); idxs.append(clip_idx); offs.append(off.to(DEV))
        singles.append(windq.windq_apply_plan(W, G, unit_rows, actions[-1], clip_idx, cg, offs[-1]))
        codes_b.append(torch.full((max(int(off[-1]), 16),), 0xAB, dtype=torch.uint8, device=DEV))
        outs_b.append((torch.full((U * R_u,), 7.0, device=DEV), torch.full((U * R_u,), 7.0, device=DEV)))
    got = windq.windq_apply_plan_batch(Ws, G, unit_rows, actions, idxs, cg, offs, codes_b, outs_b)
    torch.cuda.synchronize()
    for one, b, off in zip(singles, got, offs):
        total = int(off[-1])
        assert same_bits(one[0][:total], b[0][:total]) and same_bits(one[1], b[1]) and same_bits(one[2], b[2])


def test_apply_plan_batch_rejects_bad_batches(windq):
    Ws, _ = block(torch.bfloat16, [(64, 128)] * 2, 11)
    action = torch.ones(1, dtype=torch.uint8, device=DEV)
    off = torch.tensor([0, 64 * 128], dtype=torch.int64, device=DEV)
    codes = torch.zeros(64 * 128, dtype=torch.uint8, device=DEV)
    out = (torch.zeros(64, device=DEV), torch.zeros(64, device=DEV))
    args = lambda k: ([action] * k, [None] * k, None, [off] * k, [codes] * k, [out] * k)
    with pytest.raises(windq.WindqError) as e:
        windq.windq_apply_plan_batch([Ws[0]] * 9, 128, 0, *args(9))
    assert e.value.status == windq.WINDQ_EINVAL
    with pytest.raises(windq.WindqError) as e:
        windq.windq_apply_plan_batch([Ws[0], Ws[1].float()], 128, 0, *args(2))
    assert e.value.status == windq.WINDQ_EINVAL


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_calib_stats_batch_equals_single_calls(windq, dtype):
    """Four inputs of a block (few tokens: one shared launch) and one long input (its own two launches)."""
    shapes = [(512, 4096), (512, 4096), (100, 1032), (512, 11008), (5000, 256)]
    Xs = [synth.activations_llm(t, c, seed=181 + i, device=DEV).to(dtype) for i, (t, c) in enumerate(shapes)]
    singles = [windq.windq_calib_stats(X) for X in Xs]
    batch = windq.windq_calib_stats_batch(Xs)
    torch.cuda.synchronize()
    for one, got in zip(singles, batch):
        assert same_bits(one[0], got[0]) and same_bits(one[1], got[1])
    with pytest.raises(windq.WindqError) as e:
        windq.windq_calib_stats_batch([Xs[0]] * 9)
    assert e.value.status == windq.WINDQ_EINVAL
    with pytest.raises(windq.WindqError) as e:
        windq.windq_calib_stats_batch([Xs[0], Xs[1].float() if dtype == torch.bfloat16 else Xs[1].bfloat16()])
    assert e.value.status == windq.WINDQ_EINVAL
