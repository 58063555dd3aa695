"""The five benchmark configurations end to end, through exactly the calls bench.py times
(paper_2605_26660_amd/workload.py: the *_batch entry points, block after block, on stacks
generated in HBM), with sampled units checked against the oracle on the very bits the
device holds: features, errors / clip indices / reference energy, codes / scales / offsets,
activation scales, and Eq. 5's total over the whole plan.  Whole stacks are checked by
what holds at any size: the plan meets its budget (Eq. 1), the code stream has the length
the layout says, errors are finite and nested (8 <= 4 <= 2 bit)."""
import numpy as np
import pytest
import torch

from oracle import sampled_check as SC
from oracle import windq_oracle as O
from paper_2605_26660_amd import workload

pytestmark = [pytest.mark.gpu, pytest.mark.oracle_pool]
DEV = "cuda:0"
REL = 1e-5


def run_and_check(stack, G, picks, pool, check_all_units_sane=True):
    stack.prepare(G)
    stack.set_plan()
    cb, nw = stack.run_step()
    torch.cuda.synchronize()
    # what holds at any size
    assert nw == stack.n_weights
    assert (cb, nw) == O.effective_bits(stack.action_all.numpy(), stack.n_unit_all.numpy())
    assert cb <= stack.target_centibits * nw                                   # Eq. 1 at the target
    want_bytes = 0
    for blk in stack.blocks:
        for m in blk.mats:
            want_bytes += sum((O.bytes_per_group(int(a), G) * m.R_u + 15) // 16 * 16 for a in m.action.tolist())
    assert stack.code_bytes == want_bytes
    if check_all_units_sane:
        for blk in stack.blocks:
            for m in blk.mats:
                e = m.err
                assert bool(torch.isfinite(e).all()) and bool((e >= 0).all()) and bool((m.ref > 0).all())
                assert bool((e[:, 0] <= e[:, 1]).all()) and bool((e[:, 1] <= e[:, 3]).all())     # nested grids
                assert bool(torch.isfinite(m.feat).all())
    samples = [stack.sample(*p) for p in picks]
    res = SC.check_units(samples, pool)
    assert not res["failures"], res["failures"][:10]
    assert res["max_rel_err"] <= REL and res["codes_equal"]
    for blk in stack.blocks[:1] + stack.blocks[-1:]:
        for x in blk.xs.values():
            assert SC.check_calib(x["X"].float().cpu().numpy(), x["s"].cpu().numpy()) <= REL
    return res


def test_config1_single_layer_every_unit(windq, oracle_pool):
    stack = workload.Stack(workload.CONFIGS[1], DEV)
    picks = [(0, 0, u) for u in range(8)]
    res = run_and_check(stack, 64, picks, oracle_pool)
    assert res["units"] == 8


def test_config2_block_as_the_benchmark_runs_it(windq, oracle_pool):
    """The batched launches over all seven matrices of the 7B-shaped block at full size: three units of every
    matrix, gate / up (11008 x 4096) and down (4096 x 11008) included; every action appears among them."""
    stack = workload.Stack(workload.CONFIGS[2], DEV)
    stack.prepare(128)
    picks = stack.sample_plan(3, 0.0, seed=11)
    assert len(picks) == 21
    stack.set_plan()
    # make sure every packing format is among the sampled units
    for n, (b, i, u) in enumerate(picks):
        stack.blocks[b].mats[i].action[u] = n % 7
    res = run_and_check_with_plan(stack, 128, picks, oracle_pool)
    assert res["units"] == 21


def run_and_check_with_plan(stack, G, picks, pool):
    """As run_and_check, for a stack whose plan was edited by hand: the layout is rebuilt from the edited actions."""
    import paper_2605_26660_amd as wq
    for blk in stack.blocks:
        for m in blk.mats:
            m.action_d = m.action.to(stack.device)
            m.off = wq.windq_plan_layout(m.action, m.R_u, G)
            m.off_d = m.off.to(stack.device)
            m.codes = torch.full((max(int(m.off[-1]), 16),), 0xAB, dtype=torch.uint8, device=stack.device)
    mats = [m for blk in stack.blocks for m in blk.mats]
    stack.code_bytes = sum(int(m.off[-1]) for m in mats)
    stack.action_all = torch.cat([m.action for m in mats])
    cb, nw = stack.run_step()
    torch.cuda.synchronize()
    assert (cb, nw) == O.effective_bits(stack.action_all.numpy(), stack.n_unit_all.numpy())
    res = SC.check_units([stack.sample(*p) for p in picks], pool)
    assert not res["failures"], res["failures"][:10]
    assert res["max_rel_err"] <= REL and res["codes_equal"]
    return res


def test_config3_7b_stack_plan_at_2_bits(windq, oracle_pool):
    """32 blocks, 6.48 G weights: every matrix type of block 0 plus 1 % of the units elsewhere."""
    stack = workload.Stack(workload.CONFIGS[3], DEV)
    stack.prepare(128)
    assert stack.n_units == 8896 and stack.n_weights == 6476005376
    frac = 0.01 if oracle_pool is not None else 0.001
    picks = stack.sample_plan(1, frac, seed=33)
    res = run_and_check(stack, 128, picks, oracle_pool)
    assert res["units"] >= 7 + (80 if oracle_pool is not None else 8)
    cb, nw = windq.windq_effective_bits(stack.action_all, stack.n_unit_all)
    assert cb / (100.0 * nw) <= 2.0
    del stack
    torch.cuda.empty_cache()


def test_config4_13b_stack_plan_at_1_58_bits(windq, oracle_pool):
    """40 blocks, 12.7 G weights, plan at 1.58 bits packed to codes."""
    stack = workload.Stack(workload.CONFIGS[4], DEV)
    stack.prepare(128)
    assert stack.n_units == 13920 and stack.n_weights == 12687769600
    frac = 0.01 if oracle_pool is not None else 0.0005
    picks = stack.sample_plan(1, frac, seed=44)
    res = run_and_check(stack, 128, picks, oracle_pool)
    assert res["units"] >= 7 + (130 if oracle_pool is not None else 6)
    cb, nw = windq.windq_effective_bits(stack.action_all, stack.n_unit_all)
    assert cb / (100.0 * nw) <= 1.58
    # at 1.58 bits nothing above ternary survives unless 1-bit units pay for it
    counts = torch.bincount(stack.action_all.long(), minlength=7)
    assert int(counts[6]) > 0 and int(counts[5]) > 0
    del stack
    torch.cuda.empty_cache()


def test_config5_70b_stack_resident_both_chunk_widths(windq, oracle_pool):
    """80 blocks, 68.5 G weights (137 GB) resident, 40 clip ratios, chunk widths 64 and 128: a fixed handful of
    units per width (k/v projections are 1024 x 8192; gate/up 28672 x 8192; down 8192 x 28672)."""
    stack = workload.Stack(workload.CONFIGS[5], DEV)
    assert stack.n_weights == 68451041280
    for G in (64, 128):
        stack.prepare(G)
        assert stack.n_units == (97280 if G == 64 else 48640)
        picks = [(0, 0, 3), (0, 1, 7), (0, 4, 5), (0, 6, 11), (41, 2, 9), (79, 3, 1), (79, 6, (28672 // G) - 1)]
        res = run_and_check(stack, G, picks, oracle_pool, check_all_units_sane=(G == 128))
        assert res["units"] == 7
    del stack
    torch.cuda.empty_cache()
