"""GPU parity of windq_refine_plan (iterative scale refinement, App. "Per-unit Scale
Optimization") against the oracle: codes, scales and offsets bit for bit, errors to 1e-5."""
import numpy as np
import pytest
import torch

from oracle import windq_oracle as O
from paper_2605_26660_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
REL = 1e-5


def to_np(t):
    return t.float().cpu().numpy()


def run_case(windq, W, s, G, unit_rows, K, n_iter, ppm=0):
    cg = synth.clip_grid(K)
    mask = keep = None
    Wn, sn = to_np(W), s.cpu().numpy()
    if ppm:
        mask = windq.windq_salient_select(W, s, G, unit_rows, ppm)
        keep = O.salient_select(Wn, sn, G, unit_rows, ppm)
    err, clip_idx, ref = windq.windq_fit_score_all_bits(W, s, G, unit_rows, cg, mask=mask)
    U, R_u = windq.n_units(W.shape[0], W.shape[1], G, unit_rows)
    ci = clip_idx.cpu().numpy()
    fit = err.cpu().numpy().astype(np.float64)
    for shift in (0, 3):
        action = ((torch.arange(U) + shift) % 7).to(torch.uint8)
        off = windq.windq_plan_layout(action, R_u, G)
        poison = torch.full((max(int(off[-1]), 16),), 0xAB, dtype=torch.uint8, device=DEV)
        codes, scale, offset, e = windq.windq_refine_plan(W, s, G, unit_rows, action.to(DEV), clip_idx, cg, off.to(DEV),
                                                          n_iter, codes=poison, mask=mask)
        torch.cuda.synchronize()
        oc, osc, oof, oe = O.refine_plan(Wn, sn, G, unit_rows, action.numpy(), ci, cg.numpy(), off.numpy(), n_iter, keep=keep)
        assert np.array_equal(codes.cpu().numpy()[:int(off[-1])], oc)
        assert np.array_equal(scale.cpu().numpy().view(np.uint32), osc.view(np.uint32))
        assert np.array_equal(offset.cpu().numpy().view(np.uint32), oof.view(np.uint32))
        g = e.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(g - oe) <= REL * oe)
        # never worse than the grid fit it started from
        want_fit = np.array([0.0 if a == 0 else fit[u, a - 1] for u, a in enumerate(action.tolist())])
        assert np.all(g <= want_fit * (1 + 2 * REL))
        # and the artefact reproduces that error
        d_err, _ = windq.windq_dequant_plan(W, s, G, unit_rows, action.to(DEV), off.to(DEV), codes, scale, offset,
                                            mask=mask, want_w_hat=False)
        torch.cuda.synchronize()
        assert np.all(np.abs(d_err.cpu().numpy() - g) <= 2 * REL * g)
        if n_iter == 0:
            c0, s0, o0 = windq.windq_apply_plan(W, G, unit_rows, action.to(DEV), clip_idx, cg, off.to(DEV), mask=mask)
            torch.cuda.synchronize()
            assert torch.equal(c0[:int(off[-1])], codes[:int(off[-1])]) and torch.equal(s0, scale) and torch.equal(o0, offset)
    return g, want_fit


@pytest.mark.parametrize("R,C,G,unit_rows,K,n_iter,dtype", [
    (128, 256, 128, 0, 20, 3, torch.bfloat16), (128, 256, 128, 64, 20, 1, torch.bfloat16),
    (100, 128, 64, 50, 7, 2, torch.bfloat16), (64, 128, 64, 0, 20, 3, torch.float32),
    (24, 80, 40, 3, 5, 4, torch.bfloat16), (70, 64, 32, 0, 4, 0, torch.bfloat16), (64, 256, 256, 0, 6, 2, torch.bfloat16)])
def test_refine_plan(windq, R, C, G, unit_rows, K, n_iter, dtype):
    W = synth.weights_llm(R, C, seed=111, device=DEV, dtype=dtype)
    X = synth.activations_llm(64, C, seed=112, device=DEV)
    s, _ = windq.windq_calib_stats(X)
    run_case(windq, W, s, G, unit_rows, K, n_iter)


def test_refine_plan_under_a_protection_mask(windq):
    W = synth.weights_llm(128, 256, seed=113, device=DEV)
    X = synth.activations_llm(64, 256, seed=114, device=DEV)
    s, _ = windq.windq_calib_stats(X)
    run_case(windq, W, s, 128, 0, 8, 3, ppm=30000)
    run_case(windq, W, s, 64, 64, 8, 2, ppm=100000)


def test_refinement_lowers_the_error_of_low_bit_plans(windq):
    """2-bit plan on heavy-tailed columns: three rounds cut the grid fit's error noticeably."""
    W = synth.weights_llm(128, 512, seed=115, device=DEV)
    X = synth.activations_llm(64, 512, seed=116, device=DEV)
    s, _ = windq.windq_calib_stats(X)
    cg = synth.clip_grid(20)
    err, clip_idx, ref = windq.windq_fit_score_all_bits(W, s, 128, 0, cg)
    action = torch.full((4,), 4, dtype=torch.uint8)
    off = windq.windq_plan_layout(action, 128, 128)
    _, _, _, e3 = windq.windq_refine_plan(W, s, 128, 0, action.to(DEV), clip_idx, cg, off.to(DEV), 3)
    torch.cuda.synchronize()
    assert float(e3.double().sum()) < 0.9 * float(err[:, 3].double().sum())


def test_degenerate_groups(windq):
    W = synth.weights_llm(64, 256, seed=117, device=DEV)
    W[0:8] = 0
    W[8:16, :128] = 0.125
    W[16, :] = 1e-38
    W[17, :128] = torch.linspace(-1, 1, 128, device=DEV).to(torch.bfloat16)
    s = torch.ones(256, device=DEV)
    run_case(windq, W, s, 128, 0, 4, 3)
