"""GPU parity at the full matrix sizes of the LLaMA-13B- and LLaMA-2-70B-shaped configs
(and the 128 x G tile units of the 7B config), in the launch configuration the benchmark
times.  The oracle cannot afford whole matrices, so it checks sampled units on the very
bits generated on the device; what holds at any size (code-stream length, Eq. 5 totals)
is checked in full."""
import numpy as np
import pytest
import torch

from oracle import windq_oracle as O
from paper_2605_26660_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
REL = 1e-5


def rel_err(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return np.max(np.abs(got - want) / (np.abs(want) + 1e-300))


def run_case(windq, rows, cols, G, K, unit_rows, seed, chunks, row_blocks):
    """chunks / row_blocks: which column chunks and row blocks the oracle samples."""
    W = synth.weights_llm(rows, cols, seed=seed, device=DEV)
    X = synth.activations_llm(512, cols, seed=seed + 1, device=DEV)
    cg = synth.clip_grid(K)
    U, R_u = windq.n_units(rows, cols, G, unit_rows)
    n_chunks = cols // G
    s, _ = windq.windq_calib_stats(X)
    feat = windq.windq_unit_features(W, s, G, unit_rows)
    err, clip_idx, ref = windq.windq_fit_score_all_bits(W, s, G, unit_rows, cg)
    action = synth.random_plan(U, R_u * G, 200, seed=seed + 2)
    units = [rb * n_chunks + j for rb in row_blocks for j in chunks]
    for i, u in enumerate(units):                      # make sure every packing format is sampled
        action[u] = 1 + (i % 6)
    off = windq.windq_plan_layout(action, R_u, G)
    codes, scale, offset = windq.windq_apply_plan(W, G, unit_rows, action.to(DEV), clip_idx, cg, off.to(DEV))
    cb, nw = windq.windq_effective_bits(action, torch.full((U,), R_u * G, dtype=torch.int64))
    torch.cuda.synchronize()

    # properties that hold at any size
    assert nw == rows * cols
    assert cb == int(sum(O.ACTION_CENTIBITS[int(a)] for a in action)) * R_u * G
    assert int(off[-1]) == sum((O.bytes_per_group(int(a), G) * R_u + 15) // 16 * 16 for a in action)
    g_err, g_ref, g_feat = err.cpu().numpy(), ref.cpu().numpy(), feat.cpu().numpy()
    assert np.all(np.isfinite(g_err)) and np.all(g_err >= 0) and np.all(g_ref > 0)
    assert np.all(g_err[:, 0] <= g_err[:, 1]) and np.all(g_err[:, 1] <= g_err[:, 3])     # nested grids: 8 <= 4 <= 2 bit

    # the sampled sub-matrix: rows of the chosen row blocks x columns of the chosen chunks
    ridx = torch.cat([torch.arange(rb * R_u, (rb + 1) * R_u) for rb in row_blocks]).to(DEV)
    cidx = torch.cat([torch.arange(j * G, (j + 1) * G) for j in chunks]).to(DEV)
    Wn = W[ridx][:, cidx].float().cpu().numpy()
    sn = s[cidx].cpu().numpy()
    ur_sub = 0 if len(row_blocks) == 1 and unit_rows == 0 else R_u
    o_err, o_idx, o_ref, table = O.fit_score_all_bits(Wn, sn, G, ur_sub, cg.numpy())
    o_feat = O.unit_features(Wn, sn, G, ur_sub)
    g_idx = clip_idx.cpu().numpy()[units]
    for i, b in zip(*np.nonzero(g_idx != o_idx)):
        assert table[i, b, g_idx[i, b]] <= table[i, b].min() * (1 + 1e-9)
    assert rel_err(g_err[units], o_err) <= REL, rel_err(g_err[units], o_err)
    assert rel_err(g_ref[units], o_ref) <= REL
    n = R_u * G
    gf = g_feat[units].astype(np.float64)
    assert np.all(np.abs(gf[:, 0] - o_feat[:, 0]) <= REL * o_feat[:, 2].max())
    assert rel_err(gf[:, 1:3], o_feat[:, 1:3]) <= REL
    assert np.array_equal(np.rint(gf[:, 3:5] * n), np.rint(o_feat[:, 3:5] * n))
    assert rel_err(gf[:, 5:8], o_feat[:, 5:8]) <= REL
    # plan: codes, scales, offsets of the sampled units bit-exact
    a_sub = action[units]
    off_sub = O.plan_layout(a_sub.numpy(), R_u, G)
    o_codes, o_scale, o_offset = O.apply_plan(Wn, G, ur_sub, a_sub.numpy(), g_idx, cg.numpy(), off_sub)
    g_codes, g_scale, g_offset = codes.cpu().numpy(), scale.cpu().numpy(), offset.cpu().numpy()
    for i, u in enumerate(units):
        nbytes = int(off_sub[i + 1] - off_sub[i])
        assert np.array_equal(g_codes[int(off[u]): int(off[u]) + nbytes], o_codes[int(off_sub[i]): int(off_sub[i + 1])]), (u, int(a_sub[i]))
        assert np.array_equal(g_scale[u * R_u:(u + 1) * R_u].view(np.uint32), o_scale[i * R_u:(i + 1) * R_u].view(np.uint32))
        assert np.array_equal(g_offset[u * R_u:(u + 1) * R_u].view(np.uint32), o_offset[i * R_u:(i + 1) * R_u].view(np.uint32))


def test_7b_tile_units(windq):
    """128 x 128 tile units (the benchmark config's ~405k-unit reading): 32 x 32 = 1024 units."""
    run_case(windq, 4096, 4096, 128, 20, 128, seed=3001, chunks=[0, 7, 31], row_blocks=[0, 13, 31])


@pytest.mark.parametrize("name,rows,cols", [("13b.attn", 5120, 5120), ("13b.gate", 13824, 5120), ("13b.down", 5120, 13824)])
def test_13b_shapes(windq, name, rows, cols):
    run_case(windq, rows, cols, 128, 20, 0, seed=4000 + rows % 97, chunks=[1, cols // 128 - 1], row_blocks=[0])


@pytest.mark.parametrize("name,rows,cols,G", [("70b.kv", 1024, 8192, 64), ("70b.kv", 1024, 8192, 128),
                                              ("70b.gate", 28672, 8192, 64), ("70b.down", 8192, 28672, 128)])
def test_70b_shapes_40_point_grid(windq, name, rows, cols, G):
    run_case(windq, rows, cols, G, 40, 0, seed=5000 + G + rows % 89, chunks=[cols // G // 2], row_blocks=[0])


def test_70b_tile_units(windq):
    run_case(windq, 8192, 8192, 64, 40, 128, seed=5555, chunks=[0, 127], row_blocks=[0, 63])
