"""Seeded synthetic inputs shaped like the paper's workloads.

These stand in for LLaMA-shaped linear weights and for calibration activations of
an instruction-tuning corpus (the paper calibrates on 64 samples x 256 tokens,
Sec. 4.1); neither exists here.  This module only draws random numbers and lays
out shapes: none of the method's arithmetic lives here, which is why both the
HIP path's harness and the oracle's tests may use it.

Every generator takes a torch device, so the same recipe runs on the host for
CPU tests and directly in HBM for full-size runs (where the oracle is then
handed copies of the very bits that were generated).
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class MatrixSpec:
    name: str
    rows: int      # output features
    cols: int      # input features (the axis activation scales live on)
    x_key: str     # which calibration activation feeds it


def block_shapes(hidden: int, ffn: int, kv: int | None = None):
    """The seven linear projections of one decoder block, in the order
    q, k, v, o, gate, up, down (weights are [out x in])."""
    kv = hidden if kv is None else kv
    return [
        MatrixSpec("attn.q", hidden, hidden, "h"),
        MatrixSpec("attn.k", kv, hidden, "h"),
        MatrixSpec("attn.v", kv, hidden, "h"),
        MatrixSpec("attn.o", hidden, hidden, "o"),
        MatrixSpec("mlp.gate", ffn, hidden, "m"),
        MatrixSpec("mlp.up", ffn, hidden, "m"),
        MatrixSpec("mlp.down", hidden, ffn, "d"),
    ]


MODEL_SHAPES = {
    "llama-7b": dict(hidden=4096, ffn=11008, kv=None, blocks=32),
    "llama-13b": dict(hidden=5120, ffn=13824, kv=None, blocks=40),
    "llama2-70b": dict(hidden=8192, ffn=28672, kv=1024, blocks=80),
}


def clip_grid(K: int, lo: float = 0.5, hi: float = 1.0) -> torch.Tensor:
    """K clip ratios evenly spaced in [lo, hi], ascending, as fp32 (host tensor)."""
    if K == 1:
        return torch.tensor([hi], dtype=torch.float32)
    k = torch.arange(K, dtype=torch.float64)
    return (lo + (hi - lo) * k / (K - 1)).to(torch.float32)


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def weights_small(rows=512, cols=512, n_outlier=4, seed=0, device="cpu", dtype=torch.float32):
    """Small single-layer case: i.i.d. N(0, 0.02^2) with a few input columns x10."""
    g = _gen(seed, device)
    W = 0.02 * torch.randn(rows, cols, generator=g, device=device, dtype=torch.float32)
    idx = torch.randperm(cols, generator=g, device=device)[:n_outlier]
    W[:, idx] *= 10.0
    return W.to(dtype).contiguous()


def activations_small(tokens=256, cols=512, seed=0, device="cpu", dtype=torch.float32):
    """Calibration activations N(0,1) with per-channel scales log-uniform in [0.1, 10]."""
    g = _gen(seed + 7919, device)
    log_scale = 2.0 * torch.rand(cols, generator=g, device=device) - 1.0
    X = torch.randn(tokens, cols, generator=g, device=device) * (10.0 ** log_scale)[None, :]
    return X.to(dtype).contiguous()


def weights_llm(rows, cols, seed, device="cpu", dtype=torch.bfloat16, heavy_frac=0.01):
    """LLM-shaped weight: N(0, 0.02^2); a fraction of the input channels is instead
    drawn Student-t (3 degrees of freedom) and scaled x5."""
    g = _gen(seed, device)
    W = torch.randn(rows, cols, generator=g, device=device, dtype=torch.float32)
    n_heavy = max(1, int(round(heavy_frac * cols)))
    idx = torch.randperm(cols, generator=g, device=device)[:n_heavy]
    z = torch.randn(rows, n_heavy, generator=g, device=device)
    chi = torch.randn(rows, n_heavy, 3, generator=g, device=device).pow(2).sum(-1) / 3.0
    W[:, idx] = 5.0 * z / chi.sqrt()
    W *= 0.02
    return W.to(dtype).contiguous()


def activations_llm(tokens, cols, seed, device="cpu", dtype=torch.bfloat16, massive_frac=0.01):
    """Calibration activations with heavy-tailed per-channel scales: log-normal
    scales, and a small fraction of 'massive' channels a further x30."""
    g = _gen(seed + 104729, device)
    scale = torch.exp(torch.randn(cols, generator=g, device=device))
    n_massive = max(1, int(round(massive_frac * cols)))
    idx = torch.randperm(cols, generator=g, device=device)[:n_massive]
    scale[idx] *= 30.0
    X = torch.randn(tokens, cols, generator=g, device=device) * scale[None, :]
    return X.to(dtype).contiguous()


def matrix_seed(config: int, layer: int, matrix_index: int) -> int:
    return 1000 * config + 8 * layer + matrix_index


# Action mix of the trained policy reported for the 8B model (Fig. 2): 39.15 % 1-bit,
# 36.54 % 1.58-bit, 15.65 % 2-bit, and 8.65 % at 3 bits or more (split evenly here
# over 3, 4, 8 and skip).  Index order follows Eq. 3: skip, 8, 4, 3, 2, 1.58, 1.
POLICY_MIX = (0.0865 / 4, 0.0865 / 4, 0.0865 / 4, 0.0865 / 4, 0.1565, 0.3654, 0.3915)
_CENTIBITS = (1600, 800, 400, 300, 200, 158, 100)


def random_plan(n_units: int, weights_per_unit, target_centibits: int, seed: int) -> torch.Tensor:
    """A random plan that meets the budget: draw actions from POLICY_MIX, then demote
    randomly chosen units one level (toward 1 bit) until the nominal total fits.
    weights_per_unit: one size for all units, or a sequence of n_units sizes (units of
    several matrices in one plan).  Returns uint8 [n_units] on the host."""
    g = _gen(seed, "cpu")
    probs = torch.tensor(POLICY_MIX, dtype=torch.float64)
    action = torch.multinomial(probs, n_units, replacement=True, generator=g).tolist()
    sizes = [int(weights_per_unit)] * n_units if isinstance(weights_per_unit, int) else [int(x) for x in weights_per_unit]
    assert len(sizes) == n_units
    total = sum(_CENTIBITS[a] * n for a, n in zip(action, sizes))
    budget = target_centibits * sum(sizes)
    order = torch.randperm(n_units, generator=g).tolist()
    i = 0
    stalled = 0
    while total > budget and stalled < n_units:
        u = order[i % n_units]
        a = action[u]
        if a < 6:
            total -= (_CENTIBITS[a] - _CENTIBITS[a + 1]) * sizes[u]
            action[u] = a + 1
            stalled = 0
        else:
            stalled += 1
        i += 1
    return torch.tensor(action, dtype=torch.uint8)
