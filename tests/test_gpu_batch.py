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


def _block_step(windq, Ws, ss, G, cg, plan, bufs):
    """features -> fit+score -> apply-plan over a block through the batch calls, into caller-owned buffers."""
    windq.windq_unit_features_batch(Ws, ss, G, 0, wss=bufs["ws"], outs=bufs["feat"])
    windq.windq_fit_score_all_bits_batch(Ws, ss, G, 0, cg, wss=bufs["ws"], outs=bufs["fit"])
    windq.windq_apply_plan_batch(Ws, G, 0, plan["action"], [f[1] for f in bufs["fit"]], cg, plan["off"], bufs["codes"],
                                 bufs["so"], wss=bufs["ws"])


def _block_buffers(windq, Ws, G, K, plan):
    bufs = {"ws": [], "feat": [], "fit": [], "codes": [], "so": []}
    for W, off in zip(Ws, plan["off_host"]):
        U, R_u = windq.n_units(W.shape[0], W.shape[1], G, 0)
        need = max(windq.workspace_bytes(c, windq.WINDQ_BF16, W.shape[0], W.shape[1], G, 0, K)
                   for c in (windq.CALL_UNIT_FEATURES, windq.CALL_FIT_SCORE, windq.CALL_APPLY_PLAN))
        bufs["ws"].append(torch.empty(need, dtype=torch.uint8, device=DEV))
        bufs["feat"].append(torch.zeros(U, 8, device=DEV))
        bufs["fit"].append((torch.zeros(U, 6, device=DEV), torch.zeros(U, 4, dtype=torch.uint8, device=DEV),
                            torch.zeros(U, device=DEV)))
        bufs["codes"].append(torch.zeros(max(int(off[-1]), 16), dtype=torch.uint8, device=DEV))
        bufs["so"].append((torch.zeros(U * R_u, device=DEV), torch.zeros(U * R_u, device=DEV)))
    return bufs


def _block_plan(windq, Ws, G):
    plan = {"action": [], "off": [], "off_host": []}
    for i, W in enumerate(Ws):
        U, R_u = windq.n_units(W.shape[0], W.shape[1], G, 0)
        action = ((torch.arange(U) + i) % 7).to(torch.uint8)
        off = windq.windq_plan_layout(action, R_u, G)
        plan["action"].append(action.to(DEV)); plan["off"].append(off.to(DEV)); plan["off_host"].append(off)
    return plan


def _flat(bufs):
    out = list(bufs["feat"]) + list(bufs["codes"])
    for f in bufs["fit"]:
        out += list(f)
    for so in bufs["so"]:
        out += list(so)
    return out


def test_block_step_on_a_side_stream(windq):
    """The calls run on the caller's stream: the same step on a second stream gives the same bits."""
    G, K = 128, 20
    Ws, ss = block(torch.bfloat16, [(256, 512), (512, 256), (192, 384)], 191)
    cg = synth.clip_grid(K)
    plan = _block_plan(windq, Ws, G)
    ref, side = _block_buffers(windq, Ws, G, K, plan), _block_buffers(windq, Ws, G, K, plan)
    _block_step(windq, Ws, ss, G, cg, plan, ref)
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        _block_step(windq, Ws, ss, G, cg, plan, side)
    st.synchronize()
    assert all(same_bits(a, b) for a, b in zip(_flat(ref), _flat(side)))


def test_block_step_replays_from_a_hip_graph(windq):
    """The library allocates nothing, never synchronises and records no memset: a step can be captured in a graph.
    Every replay, with other work on the device in between, must reproduce the eager result bit for bit."""
    G, K = 128, 20
    Ws, ss = block(torch.bfloat16, [(256, 512), (512, 256), (192, 384)], 193)
    cg = synth.clip_grid(K)
    plan = _block_plan(windq, Ws, G)
    ref, cap = _block_buffers(windq, Ws, G, K, plan), _block_buffers(windq, Ws, G, K, plan)
    _block_step(windq, Ws, ss, G, cg, plan, ref)
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        _block_step(windq, Ws, ss, G, cg, plan, cap)            # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(st)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=st):
        _block_step(windq, Ws, ss, G, cg, plan, cap)
    torch.cuda.synchronize()
    for rep in range(3):
        for t in _flat(cap):
            t.fill_(1 if t.dtype == torch.uint8 else 3.0)          # poison: the replay must rewrite everything
        _block_step(windq, Ws, ss, G, cg, plan, ref)              # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert all(same_bits(a, b) for a, b in zip(_flat(ref), _flat(cap))), rep


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_masked_batches_equal_single_prot_calls(windq, dtype):
    G, K, ppm = 128, 7, 30000
    Ws, ss = block(dtype, [(256, 512), (1024, 256), (200, 384)], 201)
    cg = synth.clip_grid(K)
    masks = [windq.windq_salient_select(W, s, G, 0, ppm) for W, s in zip(Ws, ss)]
    singles = [windq.windq_fit_score_all_bits(W, s, G, 0, cg, mask=m) for W, s, m in zip(Ws, ss, masks)]
    batch = windq.windq_fit_score_all_bits_batch(Ws, ss, G, 0, cg, masks=masks)
    torch.cuda.synchronize()
    for one, got in zip(singles, batch):
        assert all(same_bits(a, b) for a, b in zip(one, got))
    plan = _block_plan(windq, Ws, G)
    ones, codes_b, outs_b = [], [], []
    for W, m, a, off, f in zip(Ws, masks, plan["action"], plan["off"], singles):
        U, R_u = windq.n_units(W.shape[0], W.shape[1], G, 0)
        ones.append(windq.windq_apply_plan(W, G, 0, a, f[1], cg, off, mask=m))
        codes_b.append(torch.full((max(int(off[-1]), 16),), 0xAB, dtype=torch.uint8, device=DEV))
        outs_b.append((torch.full((U * R_u,), 7.0, device=DEV), torch.full((U * R_u,), 7.0, device=DEV)))
    got = windq.windq_apply_plan_batch(Ws, G, 0, plan["action"], [f[1] for f in singles], cg, plan["off"], codes_b, outs_b,
                                       masks=masks)
    torch.cuda.synchronize()
    for one, b, off in zip(ones, got, plan["off"]):
        total = int(off[-1])
        assert same_bits(one[0][:total], b[0][:total]) and same_bits(one[1], b[1]) and same_bits(one[2], b[2])
    with pytest.raises(windq.WindqError) as e:                     # a mask in every item or in none
        windq.windq_fit_score_all_bits_batch(Ws, ss, G, 0, cg, masks=[masks[0], None, masks[2]])
    assert e.value.status == windq.WINDQ_EINVAL


# ------------------------------------------------ features + fit+score from one read of W
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("G,unit_rows,K,shapes", [
    (128, 0, 20, [(256, 512), (1024, 256), (64, 128), (200, 384), (2048, 128), (192, 640), (512, 512)]),
    (64, 64, 7, [(128, 256), (64, 64), (320, 192)]),
    (8, 0, 3, [(16, 24), (8, 8)]),
    (512, 0, 5, [(72, 1024)]),
    (256, 100, 40, [(300, 256)]),
    (128, 0, 21, [(256, 256), (100, 128)]),        # two clip passes on one wavefront of a tile, one on the others
    (64, 64, 64, [(128, 128)]),                    # the largest grid
])
def test_fused_features_fit_score_equals_the_separate_calls(windq, dtype, G, unit_rows, K, shapes):
    """windq_features_fit_score(_batch) takes the first pass of the unit features out of the fit+score kernel's tiles:
    every output must be, bit for bit, what windq_unit_features and windq_fit_score_all_bits give."""
    Ws, ss = block(dtype, shapes, 171)
    Ws[0][:, :G] = 0                      # a chunk of zeros: |w| < 1e-6 everywhere, P99 = 0
    Ws[-1][0, 0] = 3.0                    # |w| >= 2: the upper half of the first-digit histogram
    cg = synth.clip_grid(K)
    feats = [windq.windq_unit_features(W, s, G, unit_rows) for W, s in zip(Ws, ss)]
    fits = [windq.windq_fit_score_all_bits(W, s, G, unit_rows, cg) for W, s in zip(Ws, ss)]
    one = [windq.windq_features_fit_score(W, s, G, unit_rows, cg) for W, s in zip(Ws, ss)]
    batch = windq.windq_features_fit_score_batch(Ws, ss, G, unit_rows, cg)
    torch.cuda.synchronize()
    for f, (e, c, r), o, b in zip(feats, fits, one, batch):
        for want, got1, got2 in zip((f, e, c, r), o, b):
            assert same_bits(want, got1) and same_bits(want, got2)


def test_fused_call_checks_its_arguments(windq):
    Ws, ss = block(torch.bfloat16, [(64, 128)] * 2, 9)
    cg = synth.clip_grid(4)
    small = [torch.empty(windq.workspace_bytes(windq.CALL_FIT_SCORE, windq.WINDQ_BF16, 64, 128, 128, 0, 4), dtype=torch.uint8,
                         device=DEV)] * 2
    with pytest.raises(windq.WindqError) as e:
        windq.windq_features_fit_score_batch(Ws, ss, 128, 0, cg, wss=small)        # fit+score's size alone is too small
    assert e.value.status == windq.WINDQ_EWORKSPACE
    with pytest.raises(windq.WindqError) as e:
        windq.windq_features_fit_score_batch(Ws, ss, 96, 0, cg)
    assert e.value.status == windq.WINDQ_ESHAPE
    need = windq.workspace_bytes(windq.CALL_FEATURES_FIT_SCORE, windq.WINDQ_BF16, 64, 128, 128, 0, 4)
    assert need == (windq.workspace_bytes(windq.CALL_UNIT_FEATURES, windq.WINDQ_BF16, 64, 128, 128, 0, 4) +
                    windq.workspace_bytes(windq.CALL_FIT_SCORE, windq.WINDQ_BF16, 64, 128, 128, 0, 4))


def test_kernel_timer_brackets_the_main_fit_score_kernel(windq):
    Ws, ss = block(torch.bfloat16, [(512, 512), (256, 384)], 19)
    cg = synth.clip_grid(20)
    windq.windq_kernel_timer(True)
    a = windq.windq_fit_score_all_bits_batch(Ws, ss, 128, 0, cg)
    windq.windq_features_fit_score(Ws[0], ss[0], 128, 0, cg)
    windq.windq_unit_features(Ws[0], ss[0], 128, 0)                  # no fit+score kernel in this one
    ms, n = windq.windq_kernel_timer_read()
    assert n == 2 and 0.0 < ms < 100.0
    assert windq.windq_kernel_timer_read() == (0.0, 0)              # read forgets
    windq.windq_kernel_timer(False)
    b = windq.windq_fit_score_all_bits_batch(Ws, ss, 128, 0, cg)
    torch.cuda.synchronize()
    assert windq.windq_kernel_timer_read() == (0.0, 0)
    for x, y in zip(a, b):
        assert all(same_bits(p, q) for p, q in zip(x, y))


# ------------------------------------------- protection, refinement, the way back: batch forms
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("G,unit_rows,ppm,shapes,flat_scale", [
    (128, 0, 30000, [(256, 512), (1024, 256), (64, 128), (200, 384), (2048, 128), (192, 640), (512, 512)], False),
    (128, 0, 30000, [(320, 256), (192, 128), (64, 384)], True),      # constant scale: most thresholds are shared
    (64, 64, 20000, [(128, 256), (64, 64), (320, 192)], False),
    (128, 0, 500, [(8, 128), (2048, 128), (16, 256)], False),         # the small matrices protect nothing
    (8, 4, 250000, [(16, 24), (8, 8)], False),
])
def test_salient_batches_equal_single_calls(windq, dtype, G, unit_rows, ppm, shapes, flat_scale):
    Ws, ss = block(dtype, shapes, 311)
    if flat_scale:
        ss = [torch.ones_like(s) for s in ss]
    singles = [windq.windq_salient_select(W, s, G, unit_rows, ppm) for W, s in zip(Ws, ss)]
    outs = [torch.full((W.shape[0], W.shape[1] // 8), 0xAB, dtype=torch.uint8, device=DEV) for W in Ws]
    masks = windq.windq_salient_select_batch(Ws, ss, G, unit_rows, ppm, outs=outs)
    torch.cuda.synchronize()
    for one, got in zip(singles, masks):
        assert same_bits(one, got)
    enc1 = [windq.windq_salient_encode(W, s, G, unit_rows, m, ppm) for W, s, m in zip(Ws, ss, singles)]
    encb = windq.windq_salient_encode_batch(Ws, ss, G, unit_rows, masks, ppm)
    torch.cuda.synchronize()
    for one, got in zip(enc1, encb):
        assert all(same_bits(a, b) for a, b in zip(one, got))


def test_salient_batches_check_their_arguments(windq):
    Ws, ss = block(torch.bfloat16, [(64, 128)] * 9, 7)
    with pytest.raises(windq.WindqError) as e:
        windq.windq_salient_select_batch(Ws, ss, 128, 0, 30000)                    # more than MAX_BATCH
    assert e.value.status == windq.WINDQ_EINVAL
    with pytest.raises(windq.WindqError) as e:
        windq.windq_salient_select_batch([Ws[0], Ws[1].float()], ss[:2], 128, 0, 30000)
    assert e.value.status == windq.WINDQ_EINVAL
    with pytest.raises(windq.WindqError) as e:
        windq.windq_salient_select_batch(Ws[:2], ss[:2], 128, 0, 1000001)
    assert e.value.status == windq.WINDQ_EINVAL
    small = [torch.empty(256, dtype=torch.uint8, device=DEV)] * 2
    with pytest.raises(windq.WindqError) as e:
        windq.windq_salient_select_batch(Ws[:2], ss[:2], 128, 0, 30000, wss=small)
    assert e.value.status == windq.WINDQ_EWORKSPACE
    masks = windq.windq_salient_select_batch(Ws[:2], ss[:2], 128, 0, 30000)
    with pytest.raises(windq.WindqError) as e:
        windq.windq_salient_encode_batch(Ws[:2], ss[:2], 96, 0, masks, 30000)
    assert e.value.status == windq.WINDQ_ESHAPE
    torch.cuda.synchronize()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("G,unit_rows,K,n_iter,shapes,masked", [
    (128, 0, 7, 3, [(256, 512), (1024, 256), (64, 128), (200, 384), (2048, 128), (192, 640), (512, 512)], False),
    (128, 0, 7, 2, [(256, 512), (200, 384), (64, 128)], True),
    (64, 64, 5, 4, [(128, 256), (64, 64), (320, 192)], True),
    (24, 0, 3, 1, [(16, 48), (70, 24)], False),                       # a width the lanes-per-row kernels do not take
])
def test_refine_and_dequant_batches_equal_single_calls(windq, dtype, G, unit_rows, K, n_iter, shapes, masked):
    Ws, ss = block(dtype, shapes, 401)
    cg = synth.clip_grid(K)
    ppm = 30000
    masks = [windq.windq_salient_select(W, s, G, unit_rows, ppm) if masked and i != 1 else None
             for i, (W, s) in enumerate(zip(Ws, ss))]                # masks item by item
    acts, offs, cis = [], [], []
    for i, (W, s) in enumerate(zip(Ws, ss)):
        U, R_u = windq.n_units(W.shape[0], W.shape[1], G, unit_rows)
        gen = torch.Generator().manual_seed(600 + i)
        a = torch.randint(0, 7, (U,), generator=gen, dtype=torch.uint8)
        offs.append(windq.windq_plan_layout(a, R_u, G).to(DEV))
        acts.append(a.to(DEV))
        cis.append(torch.randint(0, K, (U, 4), generator=gen, dtype=torch.uint8).to(DEV) if i != 2 else None)
    ones = [windq.windq_refine_plan(W, s, G, unit_rows, a, ci, cg, off, n_iter, mask=m)
            for W, s, a, ci, off, m in zip(Ws, ss, acts, cis, offs, masks)]
    codes_b = [torch.full((max(int(off[-1]), 16),), 0xAB, dtype=torch.uint8, device=DEV) for off in offs]
    got = windq.windq_refine_plan_batch(Ws, ss, G, unit_rows, acts, cis, cg, offs, n_iter, codes_b, masks=masks)
    torch.cuda.synchronize()
    for one, b, off in zip(ones, got, offs):
        total = int(off[-1])
        assert same_bits(one[0][:total], b[0][:total])
        assert all(same_bits(x, y) for x, y in zip(one[1:], b[1:]))
    deq1 = [windq.windq_dequant_plan(W, s, G, unit_rows, a, off, r[0], r[1], r[2], mask=m)
            for W, s, a, off, r, m in zip(Ws, ss, acts, offs, ones, masks)]
    deqb = windq.windq_dequant_plan_batch(Ws, ss, G, unit_rows, acts, offs, [r[0] for r in got], [r[1] for r in got],
                                          [r[2] for r in got], masks=masks)
    torch.cuda.synchronize()
    for one, b in zip(deq1, deqb):
        assert same_bits(one[0], b[0]) and same_bits(one[1], b[1])
    # errors only, and the reconstruction only
    errs = windq.windq_dequant_plan_batch(Ws, ss, G, unit_rows, acts, offs, [r[0] for r in got], [r[1] for r in got],
                                          [r[2] for r in got], masks=masks, want_w_hat=False)
    torch.cuda.synchronize()
    assert all(same_bits(one[0], b[0]) and b[1] is None for one, b in zip(deq1, errs))


def test_refine_and_dequant_batches_check_their_arguments(windq):
    Ws, ss = block(torch.bfloat16, [(64, 128)] * 9, 9)
    cg = synth.clip_grid(4)
    acts = [torch.full((1,), 2, dtype=torch.uint8, device=DEV) for _ in Ws]
    offs = [windq.windq_plan_layout(torch.full((1,), 2, dtype=torch.uint8), 64, 128).to(DEV) for _ in Ws]
    codes = [torch.zeros(int(off[-1]), dtype=torch.uint8, device=DEV) for off in offs]
    with pytest.raises(windq.WindqError) as e:
        windq.windq_refine_plan_batch(Ws, ss, 128, 0, acts, [None] * 9, cg, offs, 1, codes)
    assert e.value.status == windq.WINDQ_EINVAL
    with pytest.raises(windq.WindqError) as e:
        windq.windq_refine_plan_batch(Ws[:2], ss[:2], 128, 0, acts[:2], [None] * 2, cg, offs[:2], 65, codes[:2])
    assert e.value.status == windq.WINDQ_EINVAL
    with pytest.raises(windq.WindqError) as e:
        windq.windq_refine_plan_batch([Ws[0], Ws[1].float()], ss[:2], 128, 0, acts[:2], [None] * 2, cg, offs[:2], 1, codes[:2])
    assert e.value.status == windq.WINDQ_EINVAL
    sc = [torch.zeros(64, device=DEV) for _ in Ws]
    with pytest.raises(windq.WindqError) as e:
        windq.windq_dequant_plan_batch(Ws, ss, 128, 0, acts, offs, codes, sc, sc)
    assert e.value.status == windq.WINDQ_EINVAL
    with pytest.raises(windq.WindqError) as e:
        windq.windq_dequant_plan_batch(Ws[:2], ss[:2], 96, 0, acts[:2], offs[:2], codes[:2], sc[:2], sc[:2])
    assert e.value.status == windq.WINDQ_ESHAPE
    torch.cuda.synchronize()
