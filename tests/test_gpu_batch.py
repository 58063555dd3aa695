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
