"""Sampled-unit comparison of a run of the HIP library with the oracle.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (like the oracle it sits beside): the tests
and the benchmark's parity / cpu_baseline legs hand it numpy copies of what the library
read and wrote for a few units, and it recomputes those units with `windq_oracle`.  It
imports nothing of the HIP package and nothing of torch, so worker processes that run it
never touch the GPU.

A unit is checked as a matrix of its own ([R_u x G], one chunk, all rows): every output of
the hot path for a unit depends only on the unit's weights and its chunk of the activation
scale (Sec. 3.1: units are column chunks; Sec. 3.5: local fits per unit).

Bars (the same as in tests/test_gpu_parity.py): integer outputs (codes, clip indices,
counts) and stored scales / offsets bit-exact; errors, reference energy and the
floating-point features within 1e-5 relative; a clip index may differ from the oracle's
only where the oracle's own errors at the two indices tie to 1e-9.
"""
from __future__ import annotations

import time

import numpy as np

from . import windq_oracle as O

REL = 1e-5


def _rel(got, want, floor=0.0):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.max(np.abs(got - want) / (np.abs(want) + floor + 1e-300))) if got.size else 0.0


def check_unit(sample: dict) -> dict:
    """sample: Wu [R_u x G] f32 (exact input values), s_chunk [G] f32, clip_grid [K] f32,
    and what the library produced for the unit: feat [8], err [6], clip_idx [4], ref (scalar),
    action (int), codes (u8 payload of the unit, may be empty), scale [R_u], offset [R_u].
    Any of the output entries may be missing: that part is skipped.
    Returns {"max_rel_err", "exact_ok", "failures": [...], "seconds"}."""
    t0 = time.perf_counter()
    Wu = np.ascontiguousarray(sample["Wu"], dtype=np.float32)
    s = np.asarray(sample["s_chunk"], dtype=np.float32)
    cg = np.asarray(sample["clip_grid"], dtype=np.float32)
    R_u, G = Wu.shape
    n = R_u * G
    worst = 0.0
    fails = []

    if "feat" in sample:
        want = O.unit_features(Wu, s, G, 0)[0]
        got = np.asarray(sample["feat"], dtype=np.float64)
        # the mean is a sum of signed terms: its natural scale is mean|w|
        if abs(got[0] - want[0]) > REL * want[2]:
            fails.append("feat.mean")
        r = max(_rel(got[1:3], want[1:3]), _rel(got[5:8], want[5:8], floor=1e-30))
        worst = max(worst, r)
        if r > REL:
            fails.append(f"feat {r:.2e}")
        if not np.array_equal(np.rint(got[3:5] * n), np.rint(want[3:5] * n)):
            fails.append("feat counts")

    if "err" in sample:
        E, E_t, E_b, ref = O.fit_score_unit(Wu, s, cg)
        g_idx = np.asarray(sample["clip_idx"]).astype(np.int64)
        want_err = np.zeros(6)
        for b in range(4):
            k = O.argmin_clip(E[b])
            if g_idx[b] != k and not E[b, g_idx[b]] <= E[b].min() * (1 + 1e-9):
                fails.append(f"clip_idx[{b}] {g_idx[b]} != {k}")
            want_err[b] = E[b, k]
        want_err[4], want_err[5] = E_t, E_b
        r = max(_rel(sample["err"], want_err), _rel(sample["ref"], ref))
        worst = max(worst, r)
        if r > REL:
            fails.append(f"err {r:.2e}")

    if "action" in sample and "scale" in sample:
        a = int(sample["action"])
        act = np.array([a], dtype=np.uint8)
        off = O.plan_layout(act, R_u, G)
        ci = None if "clip_idx" not in sample else np.asarray(sample["clip_idx"], dtype=np.uint8)[None, :]
        o_codes, o_scale, o_offset = O.apply_plan(Wu, G, 0, act, ci, cg if ci is not None else np.ones(1, np.float32), off)
        nbytes = O.bytes_per_group(a, G) * R_u
        if not np.array_equal(np.asarray(sample["codes"], dtype=np.uint8)[:nbytes], o_codes[:nbytes]):
            fails.append("codes")
        if not np.array_equal(np.asarray(sample["scale"], dtype=np.float32).view(np.uint32), o_scale.view(np.uint32)):
            fails.append("scale")
        if not np.array_equal(np.asarray(sample["offset"], dtype=np.float32).view(np.uint32), o_offset.view(np.uint32)):
            fails.append("offset")

    return {"max_rel_err": worst, "exact_ok": not any(f in ("codes", "scale", "offset", "feat counts") or f.startswith("clip_idx")
                                                      for f in fails),
            "failures": fails, "tag": sample.get("tag", ""), "seconds": time.perf_counter() - t0}


def check_units(samples, pool=None) -> dict:
    """All samples, in the calling process or spread over a multiprocessing pool.
    -> {"units", "max_rel_err", "codes_equal", "failures": [(tag, what)], "cpu_seconds"}."""
    results = list(pool.imap(check_unit, samples, chunksize=1)) if pool is not None else [check_unit(s) for s in samples]
    failures = [(r["tag"], f) for r in results for f in r["failures"]]
    return {"units": len(results), "max_rel_err": max((r["max_rel_err"] for r in results), default=0.0),
            "codes_equal": all(r["exact_ok"] for r in results), "failures": failures,
            "cpu_seconds": sum(r["seconds"] for r in results)}


def check_calib(X: np.ndarray, s_got: np.ndarray) -> float:
    """Largest relative deviation of the library's activation scales from the oracle's."""
    want, _ = O.calib_stats(np.asarray(X, dtype=np.float32))
    return _rel(s_got, want)


def hot_path_unit(sample: dict) -> float:
    """The oracle's five calls on one unit, for timing (cpu_baseline): returns the seconds it took."""
    t0 = time.perf_counter()
    Wu = np.ascontiguousarray(sample["Wu"], dtype=np.float32)
    s = np.asarray(sample["s_chunk"], dtype=np.float32)
    cg = np.asarray(sample["clip_grid"], dtype=np.float32)
    R_u, G = Wu.shape
    a = int(sample["action"])
    O.unit_features(Wu, s, G, 0)
    err, clip_idx, ref, _ = O.fit_score_all_bits(Wu, s, G, 0, cg)
    act = np.array([a], dtype=np.uint8)
    O.apply_plan(Wu, G, 0, act, clip_idx, cg, O.plan_layout(act, R_u, G))
    O.effective_bits(act, [R_u * G])
    return time.perf_counter() - t0
