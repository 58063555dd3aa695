"""Benchmark of the whole hot path on one MI355X.

A step = one pass of all five calls (calibration statistics, unit features, fit+score at
all six bit-widths, apply a budget-feasible plan, effective-bit accounting) over every
decoder block of the configured stack, block after block, all inputs resident in HBM.
Default: configuration 3, the LLaMA-7B-shaped stack (32 blocks, 6.48 G weights in bf16,
chunk width 128, 20 clip ratios, 512 calibration tokens per input, plan at 2.0 bits).
Prints ONE JSON line.  Synthetic seeded inputs stand in for the checkpoint and the
calibration corpus.  After the timed region: the same step with an event pair around every
call, one block alone (re-timed on the same buffers: the launch-bound small case), sampled
units against the CPU oracle, and the oracle's own speed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP32_VECTOR_PEAK_TFLOPS = 157.3    # published fp32 vector peak: 256 CU x 128 lanes x 2 flop (FMA) x 2.4 GHz


def fit_score_flops_per_weight(k: int) -> int:
    """Arithmetic of the definition, FMA = 2: per (weight, clip ratio) 1 subtract + 2 for the
    clamp + 4 bit-widths x (scale 1, rounding 1, residual 2, weighted square-accumulate 3) = 31;
    plus ternary 9, binary 4, reference energy 3, group statistics 3."""
    return 31 * k + 19


def profile_value(fname: str, key: str):
    """A 'KEY = number' line of a tracked rocprofv3 summary under profiles/ (None if absent)."""
    try:
        text = open(os.path.join(ROOT, "profiles", fname)).read()
    except OSError:
        return None
    m = re.search(r"^%s\s*=\s*([-+0-9.eE]+)" % re.escape(key), text, flags=re.M)
    return float(m.group(1)) if m else None


def start_pool():
    """Worker processes for the oracle legs.  Started before anything touches the GPU (a process that has
    initialised it must not start other programs); the workers import numpy and the oracle only."""
    import multiprocessing as mp
    n = max(1, min(16, os.cpu_count() or 1))
    try:
        pool = mp.get_context("spawn").Pool(n)
        pool.map(abs, range(n))
        return pool, n
    except Exception as e:      # the oracle legs then run in this process
        print(f"bench.py: no worker pool ({e}); oracle legs run on one core", file=sys.stderr)
        return None, 1


class CallTimer:
    """HIP events on the stream the calls are enqueued on (torch's current stream), one pair per call."""

    def __init__(self, torch, only=None):
        self.torch = torch
        self.pairs = {}
        self.only = only

    def time(self, name, fn):
        if self.only is not None and name not in self.only:
            return fn()
        e0, e1 = self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)
        e0.record()
        r = fn()
        e1.record()
        self.pairs.setdefault(name, []).append((e0, e1))
        return r

    def ms(self, name):
        return [e0.elapsed_time(e1) for e0, e1 in self.pairs.get(name, [])]


def timed_steps(torch, stack, steps, warmup, per_matrix, fused=True):
    """W untimed steps, then K timed ones; only the dominant call carries events (for the roofline)."""
    for _ in range(warmup):
        stack.run_step(per_matrix=per_matrix, fused=fused)
    torch.cuda.synchronize()
    import paper_2605_26660_amd as wq
    wq.windq_kernel_timer(True)          # an event pair around every launch of the main fit+score kernel (roofline)
    t0 = time.perf_counter()
    for _ in range(steps):
        total_cb, total_n = stack.run_step(per_matrix=per_matrix, fused=fused)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kernel_ms, n_launch = wq.windq_kernel_timer_read()
    wq.windq_kernel_timer(False)
    return dt / steps * 1e3, (kernel_ms, n_launch), total_cb, total_n


def per_call_pass(torch, stack, steps, per_matrix, fused=True):
    """The same steps with an event pair around every call (the pairs stretch a step, so this pass does
    not count toward `value`).  With the fused call, "fit_score_all_bits" is windq_features_fit_score: fit+score
    with the unit features taken from the same read of W (their later passes included)."""
    timer = CallTimer(torch)
    for _ in range(steps):
        stack.run_step(timer, per_matrix=per_matrix, fused=fused)
    torch.cuda.synchronize()
    code_bytes = stack.code_bytes + stack.meta_bytes()
    call_bytes = {"calib_stats": stack.n_activations * stack.blocks[0].mats[0].W.element_size(),
                  "unit_features": stack.n_weights * stack.blocks[0].mats[0].W.element_size(),
                  "fit_score_all_bits": stack.n_weights * stack.blocks[0].mats[0].W.element_size(),
                  "apply_plan": stack.n_weights * stack.blocks[0].mats[0].W.element_size() + code_bytes}
    calls = {}
    for name, nbytes in call_bytes.items():
        ms = timer.ms(name)
        if not ms:
            continue
        n_per_step = len(ms) // steps
        steps_ms = sorted(sum(ms[i * n_per_step:(i + 1) * n_per_step]) for i in range(steps))
        med = steps_ms[len(steps_ms) // 2]
        calls[name] = {"ms_per_step_median": med, "ms_per_step_min": steps_ms[0], "launches_per_step": n_per_step,
                       "algorithmic_bytes_per_step": nbytes, "GBps": nbytes / (med * 1e-3) / 1e9,
                       "pct_hbm_peak": 100.0 * nbytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBS}
        if name != "calib_stats":
            calls[name]["units_per_s"] = stack.n_units / (med * 1e-3)
    return calls


def roofline(stack, fit_ms, steps, per_matrix, fused=True):
    """The main fit+score kernel against the fp32 vector peak: algorithmic flops of one launch / its duration
    between a pair of HIP events that the library records around that kernel alone (windq_kernel_timer), over
    the timed region.  With the fused call the kernel also makes the unit features' pass over W; its flops
    (2 per weight for the sums of w and w^2) are not counted."""
    kernel_ms, total_launches = fit_ms
    n_launch = total_launches // steps
    avg_ms = kernel_ms / total_launches
    w_per_launch = stack.n_weights / n_launch
    flops = fit_score_flops_per_weight(stack.K)
    achieved = flops * w_per_launch / (avg_ms * 1e-3) / 1e12
    es = stack.blocks[0].mats[0].W.element_size()
    # HBM bytes per launch over one 7B-shaped block, from the tracked rocprofv3 --pmc summary (not measured live)
    traffic = profile_value("hot_path_7b_block_pmc_traffic.txt", "FIT_SCORE_TRAFFIC_BYTES_PER_BLOCK_LAUNCH")
    same_shape = stack.cfg.number in (2, 3) and stack.G == 128 and not per_matrix
    return {"bound": "alu", "achieved": achieved, "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": achieved / FP32_VECTOR_PEAK_TFLOPS,
            "traffic": traffic if same_shape else None,
            "traffic_source": "profiles/hot_path_7b_block_pmc_traffic.txt (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; bytes per launch)",
            "algorithmic_bytes_per_launch": w_per_launch * es,
            "kernel": "fit_score_kernel%s, %d launch%s per step: %s" % (
                " (with the unit features' pass over W: windq_features_fit_score)" if fused else "",
                n_launch, "es" if n_launch > 1 else "", "one per matrix" if per_matrix else "one per decoder block"),
            "avg_launch_ms": avg_ms, "flops_per_weight": flops,
            "weight_GBps": w_per_launch * es / (avg_ms * 1e-3) / 1e9,
            "pct_hbm_peak": 100.0 * w_per_launch * es / (avg_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "valu_issue_frac": profile_value("fit_score_issue_counters.txt", "VALU_ISSUE_FRAC"),
            "clip_grid_knee_K": profile_value("fit_score_clip_sweep.txt", "KNEE_K")}


def one_block(torch, stack, steps, warmup, fused=True):
    """Block 0 alone, re-timed on the same buffers (405 MB of weights at the 7B shape: larger than the
    last-level cache, but the small inputs and outputs stay warm, and a launch per kernel is all there is)."""
    sub = stack.subset([0])
    ms, fit_ms, _, _ = timed_steps(torch, sub, steps, warmup, False, fused)
    es = stack.blocks[0].mats[0].W.element_size()
    fit = fit_ms[0] / fit_ms[1]
    return {"weights": sub.n_weights, "units": sub.n_units, "ms_per_step": ms, "GBps": sub.n_weights * es / (ms * 1e-3) / 1e9,
            "fit_score_kernel_ms": fit, "fit_score_GBps": sub.n_weights * es / (fit * 1e-3) / 1e9,
            "fit_score_frac_of_fp32_peak": fit_score_flops_per_weight(stack.K) * sub.n_weights / (fit * 1e-3) / 1e12 / FP32_VECTOR_PEAK_TFLOPS}


def protected_pass(wq, torch, stack, ppm, reps):
    """Block 0 with salient-weight protection at `ppm` parts per million: mask selection and INT8
    encoding, then fit+score and apply-plan under the masks, refinement and the dequantisation check: every one a
    batch call over the block's matrices.  Timed per call with events, outside the step that `value` is quoted on."""
    G, unit_rows, cg = stack.G, stack.unit_rows, stack.clip_grid
    blk = stack.blocks[0]
    mats = blk.mats
    dt = wq.WINDQ_BF16 if stack.cfg.dtype == torch.bfloat16 else wq.WINDQ_F32
    timer = CallTimer(torch)
    extra = []
    for m in mats:
        sp = m.spec
        n_p = wq.windq_n_protected(m.R_u * G, ppm)
        need = max(wq.workspace_bytes(c, dt, sp.rows, sp.cols, G, unit_rows, stack.K)
                   for c in (wq.CALL_SALIENT, wq.CALL_DEQUANT, wq.CALL_REFINE, wq.CALL_DEQUANT_GEMV))
        extra.append(dict(
            mask=torch.empty(sp.rows, sp.cols // 8, dtype=torch.uint8, device=m.W.device),
            ws=torch.empty(need, dtype=torch.uint8, device=m.W.device),
            out=(torch.empty(m.U, n_p, dtype=torch.int8, device=m.W.device),
                 torch.empty(m.U, dtype=torch.float32, device=m.W.device),
                 torch.empty(m.U, dtype=torch.float32, device=m.W.device)),
            err=torch.empty(m.U, dtype=torch.float32, device=m.W.device),
            x=torch.randn(sp.cols, device=m.W.device), y=torch.empty(sp.rows, dtype=torch.float32, device=m.W.device),
            n_prot=torch.full((m.U,), n_p, dtype=torch.int64)))
    total_cb = total_n = 0
    for rep in range(reps + 1):
        if rep == 1:
            timer = CallTimer(torch)          # the first round is the warm-up
        total_cb = total_n = 0
        Ws = [m.W for m in mats]
        ss = [blk.xs[m.spec.x_key]["s"] for m in mats]
        masks = [e["mask"] for e in extra]
        wss = [e["ws"] for e in extra]
        timer.time("salient_select", lambda: wq.windq_salient_select_batch(Ws, ss, G, unit_rows, ppm, wss=wss, outs=masks))
        timer.time("salient_encode", lambda: wq.windq_salient_encode_batch(Ws, ss, G, unit_rows, masks, ppm, wss=wss,
                                                                           outs=[e["out"] for e in extra]))
        timer.time("fit_score_all_bits_prot", lambda: wq.windq_fit_score_all_bits_batch(
            Ws, ss, G, unit_rows, cg, wss=stack.ws, outs=[(m.err, m.clip_idx, m.ref) for m in mats], masks=masks))
        timer.time("apply_plan_prot", lambda: wq.windq_apply_plan_batch(
            Ws, G, unit_rows, [m.action_d for m in mats], [m.clip_idx for m in mats], cg, [m.off_d for m in mats],
            [m.codes for m in mats], [(m.scale, m.offset) for m in mats], wss=stack.ws, masks=masks))
        timer.time("refine_plan_prot_3_rounds", lambda: wq.windq_refine_plan_batch(
            Ws, ss, G, unit_rows, [m.action_d for m in mats], [m.clip_idx for m in mats], cg, [m.off_d for m in mats], 3,
            [m.codes for m in mats], outs=[(m.scale, m.offset, e["err"]) for m, e in zip(mats, extra)], masks=masks, wss=wss))
        timer.time("dequant_plan_prot", lambda: wq.windq_dequant_plan_batch(
            Ws, ss, G, unit_rows, [m.action_d for m in mats], [m.off_d for m in mats], [m.codes for m in mats],
            [m.scale for m in mats], [m.offset for m in mats], masks=masks, wss=wss,
            outs=[(e["err"], None) for e in extra]))
        timer.time("dequant_gemv_prot", lambda: wq.windq_dequant_gemv_batch(
            Ws, G, unit_rows, [m.action_d for m in mats], [m.off_d for m in mats], [m.codes for m in mats],
            [m.scale for m in mats], [m.offset for m in mats], [e["x"] for e in extra], masks=masks, wss=wss,
            outs=[e["y"] for e in extra]))
        for m, e in zip(mats, extra):
            cb, n = wq.windq_effective_bits(m.action, m.n_unit, e["n_prot"])
            total_cb += cb
            total_n += n
    torch.cuda.synchronize()
    n_weights = sum(m.spec.rows * m.spec.cols for m in mats)
    es = mats[0].W.element_size()
    res = {"workload": "block 0 of the stack", "rate_ppm": ppm, "avg_bits": total_cb / (100.0 * total_n)}
    for name in ("salient_select", "salient_encode", "fit_score_all_bits_prot", "apply_plan_prot", "refine_plan_prot_3_rounds",
                 "dequant_plan_prot", "dequant_gemv_prot"):
        ms = timer.ms(name)
        per = len(ms) // reps
        steps = sorted(sum(ms[i * per:(i + 1) * per]) for i in range(reps))
        med = steps[len(steps) // 2]
        res[name] = {"ms_per_block_median": med, "weight_GBps": n_weights * es / (med * 1e-3) / 1e9,
                     "pct_hbm_peak": 100.0 * n_weights * es / (med * 1e-3) / 1e9 / HBM_PEAK_GBS}
    fit = res["fit_score_all_bits_prot"]["ms_per_block_median"]
    res["fit_score_all_bits_prot"]["TFLOPs"] = fit_score_flops_per_weight(stack.K) * n_weights / (fit * 1e-3) / 1e12
    # the plain plan has to be back in place for the parity leg
    stack.subset([0]).run_step()
    torch.cuda.synchronize()
    return res


def clip_sweep(wq, synth, torch, stack, reps=3):
    """fit+score alone over block 0 at growing clip grids: where the call leaves the HBM roofline for the ALU one."""
    blk = stack.blocks[0]
    mats = blk.mats
    G, unit_rows = stack.G, stack.unit_rows
    dt = wq.WINDQ_BF16 if stack.cfg.dtype == torch.bfloat16 else wq.WINDQ_F32
    n_weights = sum(m.spec.rows * m.spec.cols for m in mats)
    es = mats[0].W.element_size()
    Ws = [m.W for m in mats]
    ss = [blk.xs[m.spec.x_key]["s"] for m in mats]
    outs = [(torch.empty_like(m.err), torch.empty_like(m.clip_idx), torch.empty_like(m.ref)) for m in mats]
    rows = []
    for k in (1, 2, 3, 4, 5, 6, 8, 10, 15, 20, 30, 40):
        cg = synth.clip_grid(k)
        ws = [torch.empty(wq.workspace_bytes(wq.CALL_FIT_SCORE, dt, m.spec.rows, m.spec.cols, G, unit_rows, k),
                          dtype=torch.uint8, device=m.W.device) for m in mats]
        best = None
        for _ in range(reps + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            wq.windq_fit_score_all_bits_batch(Ws, ss, G, unit_rows, cg, wss=ws, outs=outs)
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1)
            best = t if best is None else min(best, t)
        gbs = n_weights * es / (best * 1e-3) / 1e9
        rows.append({"K": k, "ms": best, "weight_GBps": gbs, "pct_hbm_peak": 100.0 * gbs / HBM_PEAK_GBS,
                     "TFLOPs": fit_score_flops_per_weight(k) * n_weights / (best * 1e-3) / 1e12})
    return rows


def parity_leg(stack, pool, n_elsewhere=3):
    """Sampled units of what the timed calls left in HBM against the oracle: two units of every matrix of block 0,
    a few units of other blocks, the activation scales of block 0, and Eq. 5 over the whole plan."""
    from oracle import sampled_check as SC
    from oracle import windq_oracle as O
    picks = stack.sample_plan(2, 0.0, seed=4242)
    if len(stack.blocks) > 1 and n_elsewhere > 0:
        n_rest = sum(m.U for blk in stack.blocks[1:] for m in blk.mats)
        picks += stack.sample_plan(0, n_elsewhere / n_rest, seed=4243)
    samples = [stack.sample(*p) for p in picks]
    res = SC.check_units(samples, pool)
    calib = max(SC.check_calib(x["X"].float().cpu().numpy(), x["s"].cpu().numpy()) for x in stack.blocks[0].xs.values())
    cb, nw = stack.run_step_totals
    o_cb, o_nw = O.effective_bits(stack.action_all.numpy(), stack.n_unit_all.numpy())
    return {"units": res["units"], "max_rel_err": max(res["max_rel_err"], calib), "codes_equal": bool(res["codes_equal"]),
            "effective_bits_equal": (cb, nw) == (o_cb, o_nw), "failures": res["failures"][:8],
            "what": "features, err/clip_idx/ref_energy, codes/scales/offsets of sampled units; activation scales of block 0; Eq. 5 total"}


def cpu_baseline(stack, pool, n_workers, n_units=64):
    """The oracle, as it stands, on a bounded sample of the same workload: the five calls on `n_units` units of
    block 0 (features, fit+score, apply-plan, bit accounting per unit; calibration statistics of the block's first
    input), once on one core and once spread over the worker processes."""
    from oracle import sampled_check as SC
    from oracle import windq_oracle as O
    picks = stack.sample_plan(max(1, (n_units + len(stack.specs) - 1) // len(stack.specs)), 0.0, seed=99)[:n_units]
    samples = [stack.sample(*p) for p in picks]
    n_w = sum(s["Wu"].size for s in samples)
    es = stack.blocks[0].mats[0].W.element_size()
    X = next(iter(stack.blocks[0].xs.values()))["X"].float().cpu().numpy()
    t0 = time.perf_counter()
    O.calib_stats(X)
    t_cal = time.perf_counter() - t0
    t0 = time.perf_counter()
    for s in samples:
        SC.hot_path_unit(s)
    t1 = time.perf_counter() - t0 + t_cal
    one = {"value": n_w * es / t1 / 1e9, "unit": "GB/s", "cores": 1, "seconds": t1}
    out = {"value": one["value"], "unit": "GB/s", "cores": 1, "kind": "oracle", "seconds": t1, "host_cpu_count": os.cpu_count(),
           "sample": f"{len(samples)} units of block 0 ({n_w} weights), all five calls per unit", "one_core": one}
    if pool is not None and n_workers > 1:
        t0 = time.perf_counter()
        list(pool.imap_unordered(SC.hot_path_unit, samples, chunksize=1))
        tn = time.perf_counter() - t0 + t_cal
        out.update({"value": n_w * es / tn / 1e9, "cores": min(n_workers, len(samples)), "seconds": tn})
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, choices=(1, 2, 3, 4, 5),
                    help="1 single fp32 layer; 2 one 7B block; 3 the 32-block 7B stack (default); 4 13B stack; 5 70B stack")
    ap.add_argument("--blocks", type=int, default=None, help="fewer blocks than the configuration has (for quick runs)")
    ap.add_argument("--chunk-w", type=int, default=None, help="one chunk width (configuration 5 runs 64 and 128 by default)")
    ap.add_argument("--unit-rows", type=int, default=0, help="0 = the paper's units (all rows); 128 = 128 x G tiles")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true")
    ap.add_argument("--per-matrix", action="store_true",
                    help="one call per matrix instead of the *_batch entry points (one call per kernel and block)")
    ap.add_argument("--separate-features", action="store_true",
                    help="windq_unit_features and windq_fit_score_all_bits as two calls (W read twice more) instead of "
                         "windq_features_fit_score")
    ap.add_argument("--protect-ppm", type=int, default=30000,
                    help="also time block 0 under salient-weight protection at this rate (parts per million; 0 = skip)")
    ap.add_argument("--clip-sweep", action="store_true",
                    help="also time fit+score alone over block 0 at 1..40 clip ratios (where it leaves the HBM roofline)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run plain device copies of 1 GiB (calibrates the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    want_oracle = not (args.no_cpu_baseline and args.no_parity)
    pool, n_workers = start_pool() if want_oracle else (None, 1)

    import torch

    import paper_2605_26660_amd as wq
    from paper_2605_26660_amd import synth, workload

    wq.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; libwindq has no CPU path", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = workload.CONFIGS[args.config]
    t_build = time.perf_counter()
    stack = workload.Stack(cfg, dev, n_blocks=args.blocks)
    torch.cuda.synchronize()
    t_build = time.perf_counter() - t_build

    if args.copy_probe:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    widths = (args.chunk_w,) if args.chunk_w else cfg.chunk_ws
    per_width = {}
    for G in widths:
        stack.prepare(G, args.unit_rows)
        stack.set_plan()
        fused = not args.separate_features
        ms_per_step, fit_ms, total_cb, total_n = timed_steps(torch, stack, args.steps, args.warmup, args.per_matrix, fused)
        stack.run_step_totals = (total_cb, total_n)
        es = stack.blocks[0].mats[0].W.element_size()
        r = {
            "chunk_w": G, "ms_per_step": ms_per_step, "GBps": stack.n_weights * es / (ms_per_step * 1e-3) / 1e9,
            "units": stack.n_units, "units_per_s": stack.n_units / (ms_per_step * 1e-3),
            "avg_bits": total_cb / (100.0 * total_n), "target_bits": stack.target_centibits / 100.0,
            "budget_met": total_cb <= stack.target_centibits * total_n,
            "packed_code_bytes": stack.code_bytes, "scale_offset_bytes": stack.meta_bytes(),
            "roofline": roofline(stack, fit_ms, args.steps, args.per_matrix, fused),
            "calls": per_call_pass(torch, stack, max(1, min(args.steps, 5)), args.per_matrix, fused),
        }
        # units of the last block whose P99 needed the exact pass over their weights (the workspaces are
        # shared by the blocks and hold the last one's counters)
        # (fused call only: as separate calls, fit+score reuses the workspace after the features)
        if fused:
            last = stack.blocks[-1].mats
            r["features_exact_units_last_block"] = sum(
                wq.windq_unit_features_exact_units(stack.ws[i], m.W, G, stack.unit_rows) for i, m in enumerate(last))
        if len(stack.blocks) > 1 and not args.per_matrix:
            r["one_block"] = one_block(torch, stack, max(args.steps, 20), 10, fused)
        if args.protect_ppm > 0 and G == widths[-1]:
            r["protected"] = protected_pass(wq, torch, stack, args.protect_ppm, 5)
        if args.clip_sweep and G == widths[-1]:
            r["clip_sweep"] = clip_sweep(wq, synth, torch, stack)
        if not args.no_parity:
            r["parity"] = parity_leg(stack, pool)
        if not args.no_cpu_baseline and G == widths[-1]:
            r["cpu_baseline"] = cpu_baseline(stack, pool, n_workers)
        per_width[G] = r

    head = per_width[widths[-1]]
    n_blocks = len(stack.blocks)
    out = {
        "metric": "weight GB/s scored across all 6 bit-widths (units/s) + % HBM peak, 7B shape",
        "value": head["GBps"], "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == torch.bfloat16 else "f32", "data": "synthetic",
        "config": {"workload": "configs[%d] (configuration %d): %s%s, %s, chunk %d, %d clip ratios, %d calibration tokens, plan at %.2f bits; "
                               "a step = all five calls over every block in sequence" % (
                                   cfg.number - 1, cfg.number, cfg.name, "" if n_blocks == cfg.blocks else " (first %d blocks only)" % n_blocks,
                                   "bf16" if cfg.dtype == torch.bfloat16 else "fp32", head["chunk_w"], stack.K, cfg.tokens,
                                   cfg.target_centibits / 100.0),
                   "launches": "per matrix" if args.per_matrix else "batched (one launch per kernel and decoder block)",
                   "features": "separate call" if args.separate_features else "fused into fit+score (windq_features_fit_score)",
                   "weights": stack.n_weights, "blocks": n_blocks, "units": head["units"], "unit_rows": args.unit_rows,
                   "chunk_w": head["chunk_w"], "K": stack.K, "resident_weight_bytes": stack.n_weights * es,
                   "generate_seconds": t_build},
        "value_is": "whole step (all five calls); the fused fit-and-score call alone is fit_score_GBps",
        "fit_score_GBps": head["roofline"]["weight_GBps"],
        "fit_score_pct_hbm_peak": head["roofline"]["pct_hbm_peak"],
        "units_per_s": head["units_per_s"],
        "pct_hbm_peak_whole_step": 100.0 * head["GBps"] / HBM_PEAK_GBS,
        "avg_bits": head["avg_bits"], "target_bits": head["target_bits"], "budget_met": head["budget_met"],
        "packed_code_bytes": head["packed_code_bytes"], "scale_offset_bytes": head["scale_offset_bytes"],
        "calls": head["calls"], "calls_note": "separate pass after the timed region, an event pair around every call",
        "roofline": head["roofline"],
    }
    for key in ("features_exact_units_last_block", "one_block", "protected", "clip_sweep", "parity", "cpu_baseline"):
        if key in head:
            out[key] = head[key]
    if len(widths) > 1:
        out["other_chunk_widths"] = {str(G): {k: v for k, v in per_width[G].items() if k not in ("protected", "clip_sweep")}
                                     for G in widths[:-1]}
    if pool is not None:
        pool.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
