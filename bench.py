"""Benchmark of the whole hot path on one MI355X.

A step = one pass of all five calls (calibration statistics, unit features, fit+score
at all six bit-widths, apply a budget-feasible plan, effective-bit accounting) over one
LLaMA-7B-shaped decoder block in bf16 (7 projections, 202,375,168 weights, chunk width
128, 20 clip ratios, 512 calibration tokens per input), all inputs resident in HBM.
Prints ONE JSON line.  Synthetic seeded inputs stand in for the checkpoint and the
calibration corpus.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

G = 128
K = 20
TOKENS = 512
TARGET_CENTIBITS = 200
HBM_PEAK_GBS = 8000.0
FP32_VECTOR_PEAK_TFLOPS = 157.3    # published fp32 vector peak: 256 CU x 128 lanes x 2 flop (FMA) x 2.4 GHz
# HBM bytes of the 7 fit_score launches of one step, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# file, scaled by a plain copy of known size (profiles/hot_path_7b_block_pmc_traffic.txt).  Not measured live.
FIT_SCORE_TRAFFIC_BYTES_PER_STEP = 423.7e6


def fit_score_flops_per_weight(k: int) -> int:
    """Arithmetic of the definition, FMA = 2: per (weight, clip ratio) 1 subtract + 2 for the
    clamp + 4 bit-widths x (scale 1, rounding 1, residual 2, weighted square-accumulate 3) = 31;
    plus ternary 9, binary 4, reference energy 3, group statistics 3."""
    return 31 * k + 19


def build_block(wq, synth, torch, dev, unit_rows):
    specs = synth.block_shapes(4096, 11008)
    cg = synth.clip_grid(K)
    xs = {}
    for key, cols in (("h", 4096), ("o", 4096), ("m", 4096), ("d", 11008)):
        X = synth.activations_llm(TOKENS, cols, seed=synth.matrix_seed(2, 0, len(xs)), device=dev)
        xs[key] = dict(X=X, s=torch.empty(cols, dtype=torch.float32, device=dev),
                       ws=torch.empty(wq.workspace_bytes(wq.CALL_CALIB_STATS, wq.WINDQ_BF16, TOKENS, cols),
                                      dtype=torch.uint8, device=dev))
    mats = []
    for i, sp in enumerate(specs):
        W = synth.weights_llm(sp.rows, sp.cols, seed=synth.matrix_seed(2, 0, i), device=dev)
        U, R_u = wq.n_units(sp.rows, sp.cols, G, unit_rows)
        action = synth.random_plan(U, R_u * G, TARGET_CENTIBITS, seed=100 + i)
        off = wq.windq_plan_layout(action, R_u, G)
        need = max(wq.workspace_bytes(c, wq.WINDQ_BF16, sp.rows, sp.cols, G, unit_rows, K)
                   for c in (wq.CALL_UNIT_FEATURES, wq.CALL_FIT_SCORE, wq.CALL_APPLY_PLAN, wq.CALL_DEQUANT, wq.CALL_REFINE))
        mats.append(dict(
            spec=sp, W=W, U=U, R_u=R_u, action=action, action_d=action.to(dev), off=off, off_d=off.to(dev),
            n_unit=torch.full((U,), R_u * G, dtype=torch.int64),
            feat=torch.empty(U, 8, dtype=torch.float32, device=dev),
            err=torch.empty(U, 6, dtype=torch.float32, device=dev),
            clip_idx=torch.empty(U, 4, dtype=torch.uint8, device=dev),
            ref=torch.empty(U, dtype=torch.float32, device=dev),
            codes=torch.empty(max(int(off[-1]), 16), dtype=torch.uint8, device=dev),
            scale=torch.empty(U * R_u, dtype=torch.float32, device=dev),
            offset=torch.empty(U * R_u, dtype=torch.float32, device=dev),
            ws=torch.empty(need, dtype=torch.uint8, device=dev)))
    return specs, cg, xs, mats


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


class NoTimer:
    def time(self, name, fn):
        return fn()


def run_step(wq, torch, cg, xs, mats, unit_rows, timer=NoTimer(), per_matrix=False):
    """One pass of the whole hot path over the block.  By default the three per-matrix calls go through their
    *_batch entry points (one launch per kernel over the block's seven matrices, the same results bit for bit);
    per_matrix=True makes one call per matrix instead.  (calib_stats likewise: its four inputs in one launch.)"""
    if per_matrix:
        for x in xs.values():
            timer.time("calib_stats", lambda: wq.windq_calib_stats(x["X"], want_rms=False, ws=x["ws"], out=x["s"]))
        for m in mats:
            s = xs[m["spec"].x_key]["s"]
            timer.time("unit_features", lambda: wq.windq_unit_features(m["W"], s, G, unit_rows, ws=m["ws"], out=m["feat"]))
            timer.time("fit_score_all_bits", lambda: wq.windq_fit_score_all_bits(
                m["W"], s, G, unit_rows, cg, ws=m["ws"], out=(m["err"], m["clip_idx"], m["ref"])))
            timer.time("apply_plan", lambda: wq.windq_apply_plan(
                m["W"], G, unit_rows, m["action_d"], m["clip_idx"], cg, m["off_d"], codes=m["codes"], ws=m["ws"],
                out=(m["scale"], m["offset"])))
    else:
        xl = list(xs.values())
        timer.time("calib_stats", lambda: wq.windq_calib_stats_batch(
            [x["X"] for x in xl], want_rms=False, wss=[x["ws"] for x in xl], outs=[x["s"] for x in xl]))
        Ws = [m["W"] for m in mats]
        ss = [xs[m["spec"].x_key]["s"] for m in mats]
        wss = [m["ws"] for m in mats]
        timer.time("unit_features", lambda: wq.windq_unit_features_batch(
            Ws, ss, G, unit_rows, wss=wss, outs=[m["feat"] for m in mats]))
        timer.time("fit_score_all_bits", lambda: wq.windq_fit_score_all_bits_batch(
            Ws, ss, G, unit_rows, cg, wss=wss, outs=[(m["err"], m["clip_idx"], m["ref"]) for m in mats]))
        timer.time("apply_plan", lambda: wq.windq_apply_plan_batch(
            Ws, G, unit_rows, [m["action_d"] for m in mats], [m["clip_idx"] for m in mats], cg,
            [m["off_d"] for m in mats], [m["codes"] for m in mats], [(m["scale"], m["offset"]) for m in mats], wss=wss))
    total_cb = total_n = 0
    for m in mats:
        cb, n = wq.windq_effective_bits(m["action"], m["n_unit"])
        total_cb += cb
        total_n += n
    return total_cb, total_n


def protected_pass(wq, torch, cg, xs, mats, unit_rows, ppm, reps):
    """The same block with salient-weight protection at `ppm` parts per million: mask selection and INT8
    encoding once per matrix, then fit+score and apply-plan under the masks (batch calls), refinement and the
    dequantisation check per matrix.  Timed per call with events, outside the step that `value` is quoted on."""
    timer = CallTimer(torch)
    extra = []
    for m in mats:
        sp = m["spec"]
        n_p = wq.windq_n_protected(m["R_u"] * G, ppm)
        extra.append(dict(
            mask=torch.empty(sp.rows, sp.cols // 8, dtype=torch.uint8, device=m["W"].device),
            ws=torch.empty(wq.workspace_bytes(wq.CALL_SALIENT, wq.WINDQ_BF16, sp.rows, sp.cols, G, unit_rows),
                           dtype=torch.uint8, device=m["W"].device),
            out=(torch.empty(m["U"], max(n_p, 1), dtype=torch.int8, device=m["W"].device),
                 torch.empty(m["U"], dtype=torch.float32, device=m["W"].device),
                 torch.empty(m["U"], dtype=torch.float32, device=m["W"].device)),
            n_prot=torch.full((m["U"],), n_p, dtype=torch.int64)))
    total_cb = total_n = 0
    for rep in range(reps + 1):
        if rep == 1:
            timer = CallTimer(torch)          # the first round is the warm-up
        total_cb = total_n = 0
        for m, e in zip(mats, extra):
            s = xs[m["spec"].x_key]["s"]
            timer.time("salient_select", lambda: wq.windq_salient_select(m["W"], s, G, unit_rows, ppm, ws=e["ws"], out=e["mask"]))
            timer.time("salient_encode", lambda: wq.windq_salient_encode(m["W"], s, G, unit_rows, e["mask"], ppm, ws=e["ws"], out=e["out"]))
        # fit+score and apply-plan under the masks: the block in one launch each
        Ws = [m["W"] for m in mats]
        ss = [xs[m["spec"].x_key]["s"] for m in mats]
        wss = [m["ws"] for m in mats]
        masks = [e["mask"] for e in extra]
        timer.time("fit_score_all_bits_prot", lambda: wq.windq_fit_score_all_bits_batch(
            Ws, ss, G, unit_rows, cg, wss=wss, outs=[(m["err"], m["clip_idx"], m["ref"]) for m in mats], masks=masks))
        timer.time("apply_plan_prot", lambda: wq.windq_apply_plan_batch(
            Ws, G, unit_rows, [m["action_d"] for m in mats], [m["clip_idx"] for m in mats], cg, [m["off_d"] for m in mats],
            [m["codes"] for m in mats], [(m["scale"], m["offset"]) for m in mats], wss=wss, masks=masks))
        for m, e in zip(mats, extra):
            s = xs[m["spec"].x_key]["s"]
            timer.time("refine_plan_prot_3_rounds", lambda: wq.windq_refine_plan(
                m["W"], s, G, unit_rows, m["action_d"], m["clip_idx"], cg, m["off_d"], 3, codes=m["codes"], mask=e["mask"],
                ws=m["ws"]))
            timer.time("dequant_plan_prot", lambda: wq.windq_dequant_plan(
                m["W"], s, G, unit_rows, m["action_d"], m["off_d"], m["codes"], m["scale"], m["offset"], mask=e["mask"],
                want_w_hat=False, ws=m["ws"]))
            cb, n = wq.windq_effective_bits(m["action"], m["n_unit"], e["n_prot"])
            total_cb += cb
            total_n += n
    torch.cuda.synchronize()
    n_weights = sum(m["spec"].rows * m["spec"].cols for m in mats)
    res = {"rate_ppm": ppm, "avg_bits": total_cb / (100.0 * total_n)}
    for name in ("salient_select", "salient_encode", "fit_score_all_bits_prot", "apply_plan_prot", "refine_plan_prot_3_rounds",
                 "dequant_plan_prot"):
        ms = timer.ms(name)
        per = len(ms) // reps
        steps = sorted(sum(ms[i * per:(i + 1) * per]) for i in range(reps))
        med = steps[len(steps) // 2]
        res[name] = {"ms_per_block_median": med, "weight_GBps": n_weights * 2 / (med * 1e-3) / 1e9,
                     "pct_hbm_peak": 100.0 * n_weights * 2 / (med * 1e-3) / 1e9 / HBM_PEAK_GBS}
    fit = res["fit_score_all_bits_prot"]["ms_per_block_median"]
    res["fit_score_all_bits_prot"]["TFLOPs"] = fit_score_flops_per_weight(K) * n_weights / (fit * 1e-3) / 1e12
    return res


def clip_sweep(wq, synth, torch, mats, xs, unit_rows, reps=3):
    """fit+score alone at growing clip grids: where the call leaves the HBM roofline for the ALU one."""
    n_weights = sum(m["spec"].rows * m["spec"].cols for m in mats)
    rows = []
    for k in (1, 2, 3, 5, 10, 20, 40):
        cg = synth.clip_grid(k)
        ws = [torch.empty(wq.workspace_bytes(wq.CALL_FIT_SCORE, wq.WINDQ_BF16, m["spec"].rows, m["spec"].cols, G, unit_rows, k),
                          dtype=torch.uint8, device=m["W"].device) for m in mats]
        best = None
        for _ in range(reps + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for m, w in zip(mats, ws):
                wq.windq_fit_score_all_bits(m["W"], xs[m["spec"].x_key]["s"], G, unit_rows, cg, ws=w,
                                            out=(m["err"], m["clip_idx"], m["ref"]))
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1)
            best = t if best is None else min(best, t)
        gbs = n_weights * 2 / (best * 1e-3) / 1e9
        rows.append({"K": k, "ms": best, "weight_GBps": gbs, "pct_hbm_peak": 100.0 * gbs / HBM_PEAK_GBS,
                     "TFLOPs": fit_score_flops_per_weight(k) * n_weights / (best * 1e-3) / 1e12})
    return rows


def cpu_baseline(torch, xs, mats, cg, unit_rows):
    """The oracle, as it stands, on a bounded sample of the same workload: the three
    4096 x 4096 projections that read the block input (attn.q, attn.k, attn.v: 96 units)
    through features, fit+score, apply-plan and bit accounting, plus the calibration
    statistics of their input."""
    from oracle import windq_oracle as O
    Xn = xs["h"]["X"].float().cpu().numpy()
    sample = mats[:3]
    host = [(m["W"].float().cpu().numpy(), m["action"].numpy(), m["R_u"]) for m in sample]
    n_w = 0
    t0 = time.perf_counter()
    s, _ = O.calib_stats(Xn)
    for Wn, action, R_u in host:
        O.unit_features(Wn, s, G, unit_rows)
        err, clip_idx, ref, _ = O.fit_score_all_bits(Wn, s, G, unit_rows, cg.numpy())
        off = O.plan_layout(action, R_u, G)
        O.apply_plan(Wn, G, unit_rows, action, clip_idx, cg.numpy(), off)
        O.effective_bits(action, [R_u * G] * len(action))
        n_w += Wn.size
    dt = time.perf_counter() - t0
    return {"value": n_w * 2 / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle", "seconds": dt,
            "sample": f"attn.q, attn.k, attn.v of the same block ({sum(m['U'] for m in sample)} units, {n_w} weights), all five calls"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--unit-rows", type=int, default=0, help="0 = the paper's units (all rows); 128 = 128 x G tiles")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-matrix", action="store_true",
                    help="one call per matrix (7 x 3 calls per step) instead of the *_batch entry points (3 calls per step)")
    ap.add_argument("--protect-ppm", type=int, default=30000,
                    help="also time the block under salient-weight protection at this rate (parts per million; 0 = skip)")
    ap.add_argument("--clip-sweep", action="store_true",
                    help="also time fit+score alone at 1..40 clip ratios (where it leaves the HBM roofline)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run plain device copies of 1 GiB (calibrates the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2605_26660_amd as wq
    from paper_2605_26660_amd import synth

    wq.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; libwindq has no CPU path", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    specs, cg, xs, mats = build_block(wq, synth, torch, dev, args.unit_rows)
    n_weights = sum(sp.rows * sp.cols for sp in specs)
    n_units = sum(m["U"] for m in mats)

    if args.copy_probe:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        run_step(wq, torch, cg, xs, mats, args.unit_rows, per_matrix=args.per_matrix)
    torch.cuda.synchronize()
    # timed region: K whole steps; only the dominant call carries events (for the roofline)
    fit_timer = CallTimer(torch, only=("fit_score_all_bits",))
    t0 = time.perf_counter()
    for _ in range(args.steps):
        total_cb, total_n = run_step(wq, torch, cg, xs, mats, args.unit_rows, fit_timer, per_matrix=args.per_matrix)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    # after it, the same steps again with an event pair around every call (the pairs cost ~7 % of a step,
    # so this pass does not count toward `value`)
    timer = CallTimer(torch)
    for _ in range(args.steps):
        run_step(wq, torch, cg, xs, mats, args.unit_rows, timer, per_matrix=args.per_matrix)
    torch.cuda.synchronize()
    n_act = sum(x["X"].numel() for x in xs.values())
    code_bytes = sum(int(m["off"][-1]) + 8 * m["U"] * m["R_u"] for m in mats)      # codes + scale/offset written
    call_bytes = {"calib_stats": n_act * 2, "unit_features": n_weights * 2, "fit_score_all_bits": n_weights * 2,
                  "apply_plan": n_weights * 2 + code_bytes}
    calls = {}
    for name, nbytes in call_bytes.items():
        ms = timer.ms(name)
        n_per_step = len(ms) // args.steps
        steps_ms = sorted(sum(ms[i * n_per_step:(i + 1) * n_per_step]) for i in range(args.steps))
        med = steps_ms[len(steps_ms) // 2]
        calls[name] = {"ms_per_step_median": med, "ms_per_step_min": steps_ms[0], "launches_per_step": n_per_step,
                       "algorithmic_bytes_per_step": nbytes, "GBps": nbytes / (med * 1e-3) / 1e9,
                       "pct_hbm_peak": 100.0 * nbytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBS}
    calls["unit_features"]["units_per_s"] = n_units / (calls["unit_features"]["ms_per_step_median"] * 1e-3)
    calls["fit_score_all_bits"]["units_per_s"] = n_units / (calls["fit_score_all_bits"]["ms_per_step_median"] * 1e-3)
    calls["apply_plan"]["units_per_s"] = n_units / (calls["apply_plan"]["ms_per_step_median"] * 1e-3)
    fit_ms = sum(fit_timer.ms("fit_score_all_bits")) / args.steps              # per step, all 7 launches
    flops = fit_score_flops_per_weight(K) * n_weights
    achieved = flops / (fit_ms * 1e-3) / 1e12
    n_fit_launches = len(mats) if args.per_matrix else 1

    out = {
        "metric": "weight GB/s scored across all 6 bit-widths (units/s) + % HBM peak, 7B shape",
        "value": n_weights * 2 / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "configs[1]: one LLaMA-7B-shaped decoder block, bf16, chunk 128, 20 clip ratios, "
                               "512 calibration tokens, plan at 2.0 bits; a step = all five calls over the block",
                   "launches": "per matrix" if args.per_matrix else "batched (one launch per kernel over the 7 matrices)",
                   "weights": n_weights, "units": n_units, "unit_rows": args.unit_rows, "chunk_w": G, "K": K},
        "units_per_s": n_units / (ms_per_step * 1e-3),
        "pct_hbm_peak_whole_step": 100.0 * n_weights * 2 / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "calls": calls, "calls_note": "separate pass after the timed region, an event pair around every call",
        "avg_bits": total_cb / (100.0 * total_n),
        "roofline": {"bound": "alu", "achieved": achieved, "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / FP32_VECTOR_PEAK_TFLOPS,
                     "traffic": FIT_SCORE_TRAFFIC_BYTES_PER_STEP / n_fit_launches,
                     "traffic_unit": "bytes per launch" + (" (mean of a step's 7)" if args.per_matrix else " (the block's 7 matrices)"),
                     "algorithmic_bytes_per_launch": n_weights * 2 / n_fit_launches,
                     "kernel": "fit_score_kernel<bf16> (+ its finalize kernel), %d launch%s per step" % (
                         n_fit_launches, "es" if n_fit_launches > 1 else ""),
                     "avg_launch_ms": fit_ms / n_fit_launches,
                     "flops_per_weight": fit_score_flops_per_weight(K)},
    }
    if args.protect_ppm > 0:
        out["protected"] = protected_pass(wq, torch, cg, xs, mats, args.unit_rows, args.protect_ppm, 5)
    if args.clip_sweep:
        out["clip_sweep"] = clip_sweep(wq, synth, torch, mats, xs, args.unit_rows)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(torch, xs, mats, cg, args.unit_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
