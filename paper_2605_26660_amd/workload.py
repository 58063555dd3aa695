"""The five benchmark configurations as stacks resident in HBM, and one pass of the hot path
over such a stack.

Harness code: it generates seeded synthetic inputs (synth.py), allocates every buffer once,
and calls the library's batch entry points block after block on the current stream.  None
of the method's arithmetic lives here.  Used by bench.py and by the GPU tests, so that what
is timed and what is checked against the oracle are the same calls on the same buffers.

Configurations (synthetic stand-ins for LLaMA-shaped checkpoints and calibration
activations; the paper's Sec. 4.1 set-up is 64 calibration samples x 256 tokens, chunk size
128-512):
  1  one 512 x 512 fp32 layer, chunk 64, 20 clip ratios, 256 calibration tokens
  2  one LLaMA-7B-shaped decoder block, bf16, chunk 128, 20 clip ratios, 512 tokens
  3  32 such blocks (6.48 G weights), then a random budget-feasible plan at 2.0 bits
  4  40 LLaMA-13B-shaped blocks (12.7 G weights), plan at 1.58 bits
  5  80 LLaMA-2-70B-shaped blocks (68.5 G weights, 137 GB), chunk 64 and 128, 40 clip ratios
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import binding as wq
from . import synth


@dataclass(frozen=True)
class Config:
    number: int
    name: str
    model: str | None        # key of synth.MODEL_SHAPES, None for the single layer
    blocks: int
    dtype: torch.dtype
    chunk_ws: tuple
    K: int
    tokens: int
    target_centibits: int


CONFIGS = {
    1: Config(1, "single 512x512 fp32 layer", None, 1, torch.float32, (64,), 20, 256, 200),
    2: Config(2, "one LLaMA-7B-shaped decoder block", "llama-7b", 1, torch.bfloat16, (128,), 20, 512, 200),
    3: Config(3, "LLaMA-7B-shaped stack, 32 blocks", "llama-7b", 32, torch.bfloat16, (128,), 20, 512, 200),
    4: Config(4, "LLaMA-13B-shaped stack, 40 blocks", "llama-13b", 40, torch.bfloat16, (128,), 20, 512, 158),
    5: Config(5, "LLaMA-2-70B-shaped stack, 80 blocks", "llama2-70b", 80, torch.bfloat16, (64, 128), 40, 512, 200),
}


class Mat:
    """One weight matrix of the stack with every output buffer of the hot path."""
    __slots__ = ("spec", "W", "U", "R_u", "feat", "err", "clip_idx", "ref", "action", "action_d", "off", "off_d",
                 "codes", "scale", "offset", "n_unit")


class Block:
    __slots__ = ("xs", "mats")


class Stack:
    """Weights and calibration activations of `cfg` generated layer by layer on `device` (never staged on the
    host), plus outputs and shared workspaces for chunk width G.  Workspaces are shared by all blocks: the
    calls of consecutive blocks are ordered on one stream."""

    def __init__(self, cfg: Config, device="cuda:0", n_blocks: int | None = None):
        self.cfg = cfg
        self.device = device
        self.blocks = []
        nb = cfg.blocks if n_blocks is None else n_blocks
        if cfg.model is None:
            specs = [synth.MatrixSpec("linear", 512, 512, "h")]
        else:
            m = synth.MODEL_SHAPES[cfg.model]
            specs = synth.block_shapes(m["hidden"], m["ffn"], m["kv"])
        self.specs = specs
        x_keys = []
        for sp in specs:
            if sp.x_key not in [k for k, _ in x_keys]:
                x_keys.append((sp.x_key, sp.cols))
        self.x_keys = x_keys
        for layer in range(nb):
            blk = Block()
            blk.xs = {}
            for xi, (key, cols) in enumerate(x_keys):
                if cfg.model is None:
                    X = synth.activations_small(cfg.tokens, cols, seed=0, device=device, dtype=cfg.dtype)
                else:
                    X = synth.activations_llm(cfg.tokens, cols, seed=synth.matrix_seed(cfg.number, layer, xi), device=device,
                                              dtype=cfg.dtype)
                blk.xs[key] = dict(X=X, s=torch.empty(cols, dtype=torch.float32, device=device))
            blk.mats = []
            for i, sp in enumerate(specs):
                m = Mat()
                m.spec = sp
                if cfg.model is None:
                    m.W = synth.weights_small(sp.rows, sp.cols, seed=0, device=device, dtype=cfg.dtype)
                else:
                    m.W = synth.weights_llm(sp.rows, sp.cols, seed=synth.matrix_seed(cfg.number, layer, i), device=device,
                                            dtype=cfg.dtype)
                blk.mats.append(m)
            self.blocks.append(blk)
        self.n_weights = sum(sp.rows * sp.cols for sp in specs) * nb
        self.n_activations = sum(cfg.tokens * cols for _, cols in x_keys) * nb
        dt = wq.WINDQ_BF16 if cfg.dtype == torch.bfloat16 else wq.WINDQ_F32
        self.calib_ws = {key: torch.empty(max(wq.workspace_bytes(wq.CALL_CALIB_STATS, dt, cfg.tokens, cols), 256),
                                          dtype=torch.uint8, device=device) for key, cols in x_keys}
        self.G = None

    # ------------------------------------------------------------------ outputs for one chunk width
    def prepare(self, G: int, unit_rows: int = 0, K: int | None = None):
        """(Re)allocate outputs and workspaces for chunk width G; drops those of an earlier width."""
        cfg = self.cfg
        self.G, self.unit_rows, self.K = G, unit_rows, (cfg.K if K is None else K)
        self.clip_grid = synth.clip_grid(self.K)
        dt = wq.WINDQ_BF16 if cfg.dtype == torch.bfloat16 else wq.WINDQ_F32
        dev = self.device
        self.ws = None
        for blk in self.blocks:
            for m in blk.mats:
                m.codes = m.scale = m.offset = None
        self.ws = [torch.empty(max(wq.workspace_bytes(c, dt, sp.rows, sp.cols, G, unit_rows, self.K)
                                   for c in (wq.CALL_UNIT_FEATURES, wq.CALL_FIT_SCORE, wq.CALL_APPLY_PLAN, wq.CALL_FEATURES_FIT_SCORE)),
                               dtype=torch.uint8, device=dev) for sp in self.specs]
        self.n_units = 0
        for blk in self.blocks:
            for m in blk.mats:
                sp = m.spec
                m.U, m.R_u = wq.n_units(sp.rows, sp.cols, G, unit_rows)
                m.n_unit = torch.full((m.U,), m.R_u * G, dtype=torch.int64)
                m.feat = torch.empty(m.U, 8, dtype=torch.float32, device=dev)
                m.err = torch.empty(m.U, 6, dtype=torch.float32, device=dev)
                m.clip_idx = torch.empty(m.U, 4, dtype=torch.uint8, device=dev)
                m.ref = torch.empty(m.U, dtype=torch.float32, device=dev)
                m.scale = torch.empty(m.U * m.R_u, dtype=torch.float32, device=dev)
                m.offset = torch.empty(m.U * m.R_u, dtype=torch.float32, device=dev)
                self.n_units += m.U
        self.n_groups = sum(m.U * m.R_u for blk in self.blocks for m in blk.mats)

    def set_plan(self, target_centibits: int | None = None, seed: int | None = None, per_matrix: bool = False):
        """A random budget-feasible plan (actions from the trained policy's mix, Fig. 2, then random one-level
        demotions until Eq. 1 holds at the target), drawn over all units of the stack at once (per_matrix: one
        draw per matrix, each meeting the target by itself).  Allocates the code streams."""
        cfg = self.cfg
        target = cfg.target_centibits if target_centibits is None else target_centibits
        seed = 1000 * cfg.number + 999 if seed is None else seed
        mats = [m for blk in self.blocks for m in blk.mats]
        if per_matrix:
            acts = [synth.random_plan(m.U, m.R_u * self.G, target, seed=seed + i) for i, m in enumerate(mats)]
        else:
            sizes = [m.R_u * self.G for m in mats for _ in range(m.U)]
            allact = synth.random_plan(len(sizes), sizes, target, seed=seed)
            acts, pos = [], 0
            for m in mats:
                acts.append(allact[pos:pos + m.U].contiguous())
                pos += m.U
        self.code_bytes = 0
        for m, a in zip(mats, acts):
            m.action = a
            m.action_d = a.to(self.device)
            m.off = wq.windq_plan_layout(a, m.R_u, self.G)
            m.off_d = m.off.to(self.device)
            m.codes = torch.empty(max(int(m.off[-1]), 16), dtype=torch.uint8, device=self.device)
            self.code_bytes += int(m.off[-1])
        self.action_all = torch.cat([m.action for m in mats])
        self.n_unit_all = torch.cat([m.n_unit for m in mats])
        self.target_centibits = target

    def subset(self, block_indices):
        """A view of some blocks of this stack (same buffers, same plan), e.g. one block alone."""
        sub = object.__new__(Stack)
        sub.__dict__.update(self.__dict__)
        sub.blocks = [self.blocks[i] for i in block_indices]
        mats = [m for blk in sub.blocks for m in blk.mats]
        per_block_w = sum(sp.rows * sp.cols for sp in self.specs)
        sub.n_weights = per_block_w * len(sub.blocks)
        sub.n_activations = sum(self.cfg.tokens * cols for _, cols in self.x_keys) * len(sub.blocks)
        sub.n_units = sum(m.U for m in mats)
        sub.n_groups = sum(m.U * m.R_u for m in mats)
        if getattr(self, "action_all", None) is not None:
            sub.code_bytes = sum(int(m.off[-1]) for m in mats)
            sub.action_all = torch.cat([m.action for m in mats])
            sub.n_unit_all = torch.cat([m.n_unit for m in mats])
        return sub

    # ------------------------------------------------------------------ one pass of the hot path
    def run_step(self, timer=None, per_matrix: bool = False, fused: bool = True):
        """All five calls over every block, in sequence, on the current stream.  Returns Eq. 5's (total centibits,
        total weights).  timer: object with time(name, fn) (an event pair per call) or None.  fused: unit features and
        fit+score through windq_features_fit_score (one read of W for both) instead of the two separate calls."""
        G, ur, cg = self.G, self.unit_rows, self.clip_grid
        t = timer.time if timer is not None else (lambda name, fn: fn())
        for blk in self.blocks:
            xl = list(blk.xs.items())
            mats = blk.mats
            if per_matrix:
                for key, x in xl:
                    t("calib_stats", lambda: wq.windq_calib_stats(x["X"], want_rms=False, ws=self.calib_ws[key], out=x["s"]))
                for i, m in enumerate(mats):
                    s = blk.xs[m.spec.x_key]["s"]
                    if fused:
                        t("fit_score_all_bits", lambda: wq.windq_features_fit_score(
                            m.W, s, G, ur, cg, ws=self.ws[i], out=(m.feat, m.err, m.clip_idx, m.ref)))
                    else:
                        t("unit_features", lambda: wq.windq_unit_features(m.W, s, G, ur, ws=self.ws[i], out=m.feat))
                        t("fit_score_all_bits", lambda: wq.windq_fit_score_all_bits(m.W, s, G, ur, cg, ws=self.ws[i],
                                                                                    out=(m.err, m.clip_idx, m.ref)))
                    t("apply_plan", lambda: wq.windq_apply_plan(m.W, G, ur, m.action_d, m.clip_idx, cg, m.off_d, codes=m.codes,
                                                                ws=self.ws[i], out=(m.scale, m.offset)))
                continue
            t("calib_stats", lambda: wq.windq_calib_stats_batch(
                [x["X"] for _, x in xl], want_rms=False, wss=[self.calib_ws[k] for k, _ in xl], outs=[x["s"] for _, x in xl]))
            Ws = [m.W for m in mats]
            ss = [blk.xs[m.spec.x_key]["s"] for m in mats]
            if fused:
                t("fit_score_all_bits", lambda: wq.windq_features_fit_score_batch(
                    Ws, ss, G, ur, cg, wss=self.ws, outs=[(m.feat, m.err, m.clip_idx, m.ref) for m in mats]))
            else:
                t("unit_features", lambda: wq.windq_unit_features_batch(Ws, ss, G, ur, wss=self.ws, outs=[m.feat for m in mats]))
                t("fit_score_all_bits", lambda: wq.windq_fit_score_all_bits_batch(
                    Ws, ss, G, ur, cg, wss=self.ws, outs=[(m.err, m.clip_idx, m.ref) for m in mats]))
            t("apply_plan", lambda: wq.windq_apply_plan_batch(
                Ws, G, ur, [m.action_d for m in mats], [m.clip_idx for m in mats], cg, [m.off_d for m in mats],
                [m.codes for m in mats], [(m.scale, m.offset) for m in mats], wss=self.ws))
        return wq.windq_effective_bits(self.action_all, self.n_unit_all)

    # ------------------------------------------------------------------ samples for the oracle
    def sample(self, block: int, mat: int, unit: int, tag: str | None = None) -> dict:
        """Host copies (numpy) of what the library read and wrote for one unit: the very bits in HBM."""
        blk = self.blocks[block]
        m = blk.mats[mat]
        G = self.G
        n_chunks = m.spec.cols // G
        rb, j = divmod(unit, n_chunks)
        rows = slice(rb * m.R_u, (rb + 1) * m.R_u)
        cols = slice(j * G, (j + 1) * G)
        s = blk.xs[m.spec.x_key]["s"]
        a = int(m.action[unit])
        lo = int(m.off[unit])
        nbytes = wq.windq_bytes_per_group(a, G) * m.R_u
        return {
            "tag": tag or f"block {block} {m.spec.name} unit {unit}",
            "Wu": m.W[rows, cols].float().cpu().numpy(), "s_chunk": s[cols].cpu().numpy(),
            "clip_grid": self.clip_grid.numpy(),
            "feat": m.feat[unit].cpu().numpy(), "err": m.err[unit].cpu().numpy(), "clip_idx": m.clip_idx[unit].cpu().numpy(),
            "ref": float(m.ref[unit]), "action": a, "codes": m.codes[lo:lo + nbytes].cpu().numpy(),
            "scale": m.scale[unit * m.R_u:(unit + 1) * m.R_u].cpu().numpy(),
            "offset": m.offset[unit * m.R_u:(unit + 1) * m.R_u].cpu().numpy(),
        }

    def sample_plan(self, per_block0: int, frac_elsewhere: float, seed: int, max_units: int | None = None):
        """(block, matrix, unit) triples: `per_block0` units of every matrix of block 0, plus a fraction of the units
        of the other blocks (seeded), at most max_units in all."""
        g = torch.Generator().manual_seed(seed)
        picks = []
        for i, m in enumerate(self.blocks[0].mats):
            for u in torch.randperm(m.U, generator=g)[:per_block0].tolist():
                picks.append((0, i, u))
        rest = [(b, i, m.U) for b, blk in enumerate(self.blocks) if b > 0 for i, m in enumerate(blk.mats)]
        n_rest = sum(u for _, _, u in rest)
        want = int(round(frac_elsewhere * n_rest))
        if max_units is not None:
            want = max(0, min(want, max_units - len(picks)))
        if want > 0:
            flat = torch.randperm(n_rest, generator=g)[:want].tolist()
            starts, pos = [], 0
            for b, i, u in rest:
                starts.append(pos)
                pos += u
            import bisect
            for f in sorted(flat):
                k = bisect.bisect_right(starts, f) - 1
                picks.append((rest[k][0], rest[k][1], f - starts[k]))
        return picks

    def meta_bytes(self) -> int:
        """Per-group scale + offset, 8 bytes per group: metadata Eq. 5 does not count."""
        return 8 * self.n_groups
