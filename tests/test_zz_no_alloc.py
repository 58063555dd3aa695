"""The entry point that allocates nothing: windq_fit_score_all_bits_static keeps its workspace in
an array built into the library.  Through the C ABI, against windq_fit_score_all_bits (which is
checked against the oracle elsewhere): the same bits, on two calls in a row, the second on a
smaller input (so the array still holds the first call's partial sums)."""
import ctypes

import pytest
import torch

from paper_2605_26660_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def same_bits(a, b):
    return torch.equal(a.contiguous().view(torch.uint8).flatten(), b.contiguous().view(torch.uint8).flatten())


def outputs(windq, W, G, unit_rows):
    U, _ = windq.n_units(W.shape[0], W.shape[1], G, unit_rows)
    return (torch.full((U, 6), -1.0, dtype=torch.float32, device=DEV), torch.full((U, 4), 255, dtype=torch.uint8, device=DEV),
            torch.full((U,), -1.0, dtype=torch.float32, device=DEV))


def test_static_workspace_call_matches_the_workspace_call(windq):
    G, K = 128, 20
    cg = synth.clip_grid(K)
    # big then small; the second one also has heavy rows, so the list of units scored twice is exercised
    shapes = [(4096, 1024, 0, torch.bfloat16), (512, 384, 0, torch.bfloat16), (256, 256, 64, torch.float32)]
    for i, (R, C, unit_rows, dtype) in enumerate(shapes):
        W = synth.weights_llm(R, C, seed=700 + i, device="cpu", dtype=torch.float32)
        if i == 1:
            W[64:128, :128] *= 300.0
        W = W.to(dtype).to(DEV)
        s = synth.activations_llm(64, C, seed=710 + i, device=DEV).float().abs().mean(0)
        assert windq.workspace_bytes(windq.CALL_FIT_SCORE, windq.WINDQ_BF16, R, C, G, unit_rows, K) <= windq.STATIC_SCRATCH_BYTES
        want = windq.windq_fit_score_all_bits(W, s, G, unit_rows, cg)
        out = outputs(windq, W, G, unit_rows)
        torch.cuda.synchronize()
        held, peak = torch.cuda.memory_allocated(), torch.cuda.max_memory_allocated()
        got = windq.windq_fit_score_all_bits_static(W, s, G, unit_rows, cg, out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() <= held and torch.cuda.max_memory_allocated() == peak   # torch allocated nothing
        for a, b in zip(want, got):
            assert same_bits(a, b)


def test_static_workspace_call_rejects_what_does_not_fit(windq):
    # 8192 x 16384 at chunk 128, K = 40: 128 units x 128 tiles x 212 x 8 bytes = 27.8 MB > 8 MiB
    m = windq.windq_mat(4096, windq.WINDQ_BF16, 0, 8192, 16384, 16384)
    cg = synth.clip_grid(40)
    assert windq.workspace_bytes(windq.CALL_FIT_SCORE, windq.WINDQ_BF16, 8192, 16384, 128, 0, 40) > windq.STATIC_SCRATCH_BYTES
    st = windq.lib().windq_fit_score_all_bits_static(ctypes.byref(m), 4096, 128, 0, cg.data_ptr(), 40, 4096, 4096, None, None)
    assert st == windq.WINDQ_EWORKSPACE
    # the other checks come first, as in the workspace call
    bad = windq.windq_mat(4096, windq.WINDQ_BF16, 0, 8192, 16400, 16400)
    assert windq.lib().windq_fit_score_all_bits_static(ctypes.byref(bad), 4096, 128, 0, cg.data_ptr(), 40, 4096, 4096, None, None) == windq.WINDQ_ESHAPE
