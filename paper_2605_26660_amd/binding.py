"""Thin ctypes binding over libwindq's C ABI (include/windq.h).

Argument marshalling only: torch tensors supply device memory and the current stream;
every step of the path runs in the HIP kernels.  There is no CPU fallback: if the
library is missing, or a GPU call is made without a GPU, this raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libwindq.so")

WINDQ_OK, WINDQ_EINVAL, WINDQ_ESHAPE, WINDQ_EDTYPE, WINDQ_EWORKSPACE, WINDQ_EHIP = range(6)
WINDQ_F32, WINDQ_BF16 = 0, 1
CALL_CALIB_STATS, CALL_UNIT_FEATURES, CALL_FIT_SCORE, CALL_APPLY_PLAN, CALL_SALIENT, CALL_UNIT_SALIENCY, CALL_DEQUANT, CALL_REFINE, CALL_FEATURES_FIT_SCORE, CALL_DEQUANT_GEMV = range(10)
N_ACTIONS, N_ERR, N_FEAT, MAX_CLIP, MAX_CHUNK, MAX_BATCH = 7, 6, 8, 64, 512, 8
STATIC_SCRATCH_BYTES = 8 << 20

EXPORTS = (
    "windq_calib_stats", "windq_unit_features", "windq_fit_score_all_bits", "windq_bytes_per_group",
    "windq_plan_layout", "windq_apply_plan", "windq_effective_bits", "windq_workspace_bytes",
    "windq_status_str", "windq_n_protected", "windq_salient_select", "windq_salient_encode",
    "windq_fit_score_all_bits_prot", "windq_apply_plan_prot", "windq_unit_saliency", "windq_heuristic_plan",
    "windq_fallback_promote", "windq_dequant_plan", "windq_refine_plan", "windq_fit_score_all_bits_batch",
    "windq_unit_features_batch", "windq_apply_plan_batch", "windq_calib_stats_batch", "windq_fit_score_rescored_units",
    "windq_fit_score_all_bits_static", "windq_features_fit_score", "windq_features_fit_score_batch",
    "windq_kernel_timer", "windq_kernel_timer_read", "windq_salient_select_batch", "windq_salient_encode_batch",
    "windq_refine_plan_batch", "windq_dequant_plan_batch", "windq_unit_features_exact_units",
    "windq_dequant_gemv", "windq_dequant_gemv_batch",
)


class WindqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.windq_status_str(status).decode() if _lib is not None else "?"
        super().__init__(f"{where}: status {status} ({msg})")


class windq_mat(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("dtype", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("rows", ctypes.c_int64), ("cols", ctypes.c_int64), ("ld", ctypes.c_int64)]


class windq_fit_item(ctypes.Structure):
    _fields_ = [("W", ctypes.POINTER(windq_mat)), ("s", ctypes.c_void_p), ("mask", ctypes.c_void_p),
                ("err", ctypes.c_void_p), ("clip_idx", ctypes.c_void_p), ("ref_energy", ctypes.c_void_p),
                ("ws", ctypes.c_void_p), ("ws_bytes", ctypes.c_size_t)]


class windq_fused_item(ctypes.Structure):
    _fields_ = [("W", ctypes.POINTER(windq_mat)), ("s", ctypes.c_void_p), ("feat", ctypes.c_void_p),
                ("err", ctypes.c_void_p), ("clip_idx", ctypes.c_void_p), ("ref_energy", ctypes.c_void_p),
                ("ws", ctypes.c_void_p), ("ws_bytes", ctypes.c_size_t)]


class windq_feat_item(ctypes.Structure):
    _fields_ = [("W", ctypes.POINTER(windq_mat)), ("s", ctypes.c_void_p), ("feat", ctypes.c_void_p),
                ("ws", ctypes.c_void_p), ("ws_bytes", ctypes.c_size_t)]


class windq_apply_item(ctypes.Structure):
    _fields_ = [("W", ctypes.POINTER(windq_mat)), ("mask", ctypes.c_void_p), ("action", ctypes.c_void_p),
                ("clip_idx", ctypes.c_void_p),
                ("code_off", ctypes.c_void_p), ("codes", ctypes.c_void_p), ("codes_bytes", ctypes.c_size_t),
                ("scale", ctypes.c_void_p), ("offset", ctypes.c_void_p), ("ws", ctypes.c_void_p),
                ("ws_bytes", ctypes.c_size_t)]


class windq_salient_item(ctypes.Structure):
    _fields_ = [("W", ctypes.POINTER(windq_mat)), ("s", ctypes.c_void_p), ("mask", ctypes.c_void_p),
                ("prot_codes", ctypes.c_void_p), ("prot_scale", ctypes.c_void_p), ("err_prot", ctypes.c_void_p),
                ("ws", ctypes.c_void_p), ("ws_bytes", ctypes.c_size_t)]


class windq_refine_item(ctypes.Structure):
    _fields_ = [("W", ctypes.POINTER(windq_mat)), ("s", ctypes.c_void_p), ("mask", ctypes.c_void_p),
                ("action", ctypes.c_void_p), ("clip_idx", ctypes.c_void_p), ("code_off", ctypes.c_void_p),
                ("codes", ctypes.c_void_p), ("codes_bytes", ctypes.c_size_t), ("scale", ctypes.c_void_p),
                ("offset", ctypes.c_void_p), ("err", ctypes.c_void_p), ("ws", ctypes.c_void_p),
                ("ws_bytes", ctypes.c_size_t)]


class windq_dequant_item(ctypes.Structure):
    _fields_ = [("W", ctypes.POINTER(windq_mat)), ("s", ctypes.c_void_p), ("mask", ctypes.c_void_p),
                ("action", ctypes.c_void_p), ("code_off", ctypes.c_void_p), ("codes", ctypes.c_void_p),
                ("codes_bytes", ctypes.c_size_t), ("scale", ctypes.c_void_p), ("offset", ctypes.c_void_p),
                ("err", ctypes.c_void_p), ("w_hat", ctypes.c_void_p), ("ws", ctypes.c_void_p),
                ("ws_bytes", ctypes.c_size_t)]


class windq_gemv_item(ctypes.Structure):
    _fields_ = [("W", ctypes.POINTER(windq_mat)), ("mask", ctypes.c_void_p), ("action", ctypes.c_void_p),
                ("code_off", ctypes.c_void_p), ("codes", ctypes.c_void_p), ("codes_bytes", ctypes.c_size_t),
                ("scale", ctypes.c_void_p), ("offset", ctypes.c_void_p), ("x", ctypes.c_void_p), ("y", ctypes.c_void_p),
                ("ws", ctypes.c_void_p), ("ws_bytes", ctypes.c_size_t)]


class windq_calib_item(ctypes.Structure):
    _fields_ = [("X", ctypes.POINTER(windq_mat)), ("s_absmean", ctypes.c_void_p), ("s_rms", ctypes.c_void_p),
                ("ws", ctypes.c_void_p), ("ws_bytes", ctypes.c_size_t)]


_lib = None


def load(path: str | None = None):
    """dlopen the in-tree library and declare the signatures.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2605_26660_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    c = ctypes
    vp, i32, i64, sz = c.c_void_p, c.c_int32, c.c_int64, c.c_size_t
    pm = c.POINTER(windq_mat)
    lib.windq_calib_stats.argtypes = [pm, vp, vp, vp, sz, vp]
    lib.windq_unit_features.argtypes = [pm, vp, i32, i64, vp, vp, sz, vp]
    lib.windq_fit_score_all_bits.argtypes = [pm, vp, i32, i64, vp, i32, vp, vp, vp, vp, sz, vp]
    lib.windq_bytes_per_group.argtypes = [i32, i32]
    lib.windq_bytes_per_group.restype = i64
    lib.windq_plan_layout.argtypes = [vp, i64, i64, i32, vp]
    lib.windq_apply_plan.argtypes = [pm, i32, i64, vp, vp, vp, i32, vp, vp, sz, vp, vp, vp, sz, vp]
    lib.windq_effective_bits.argtypes = [vp, vp, vp, i64, c.POINTER(i64), c.POINTER(i64)]
    lib.windq_workspace_bytes.argtypes = [i32, i32, i64, i64, i32, i64, i32]
    lib.windq_workspace_bytes.restype = sz
    u32 = c.c_uint32
    lib.windq_n_protected.argtypes = [i64, u32]
    lib.windq_n_protected.restype = i64
    lib.windq_salient_select.argtypes = [pm, vp, i32, i64, u32, vp, vp, sz, vp]
    lib.windq_salient_encode.argtypes = [pm, vp, i32, i64, vp, u32, vp, vp, vp, vp, sz, vp]
    lib.windq_fit_score_all_bits_prot.argtypes = [pm, vp, i32, i64, vp, vp, i32, vp, vp, vp, vp, sz, vp]
    lib.windq_apply_plan_prot.argtypes = [pm, i32, i64, vp, vp, vp, vp, i32, vp, vp, sz, vp, vp, vp, sz, vp]
    lib.windq_unit_saliency.argtypes = [pm, vp, i32, i64, vp, vp, sz, vp]
    lib.windq_heuristic_plan.argtypes = [vp, vp, vp, i64, i64, u32, u32, vp, c.POINTER(i64), c.POINTER(i32)]
    lib.windq_fallback_promote.argtypes = [vp, vp, vp, i64, c.c_float, c.POINTER(i64)]
    lib.windq_dequant_plan.argtypes = [pm, vp, i32, i64, vp, vp, vp, vp, sz, vp, vp, vp, vp, vp, sz, vp]
    lib.windq_refine_plan.argtypes = [pm, vp, i32, i64, vp, vp, vp, vp, i32, i32, vp, vp, sz, vp, vp, vp, vp, sz, vp]
    lib.windq_fit_score_all_bits_batch.argtypes = [c.POINTER(windq_fit_item), i32, i32, i64, vp, i32, vp]
    lib.windq_unit_features_batch.argtypes = [c.POINTER(windq_feat_item), i32, i32, i64, vp]
    lib.windq_apply_plan_batch.argtypes = [c.POINTER(windq_apply_item), i32, i32, i64, vp, i32, vp]
    lib.windq_calib_stats_batch.argtypes = [c.POINTER(windq_calib_item), i32, vp]
    lib.windq_features_fit_score.argtypes = [pm, vp, i32, i64, vp, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.windq_features_fit_score.restype = c.c_int
    lib.windq_features_fit_score_batch.argtypes = [c.POINTER(windq_fused_item), i32, i32, i64, vp, i32, vp]
    lib.windq_features_fit_score_batch.restype = c.c_int
    lib.windq_kernel_timer.argtypes = [i32]
    lib.windq_kernel_timer.restype = c.c_int
    lib.windq_kernel_timer_read.argtypes = [c.POINTER(c.c_double), c.POINTER(i64)]
    lib.windq_kernel_timer_read.restype = c.c_int
    lib.windq_fit_score_all_bits_static.argtypes = [pm, vp, i32, i64, vp, i32, vp, vp, vp, vp]
    lib.windq_fit_score_all_bits_static.restype = c.c_int
    lib.windq_fit_score_rescored_units.argtypes = [vp, i32, i64, i64, i32, i64, i32, c.POINTER(i64)]
    lib.windq_fit_score_rescored_units.restype = c.c_int
    lib.windq_salient_select_batch.argtypes = [c.POINTER(windq_salient_item), i32, i32, i64, u32, vp]
    lib.windq_salient_select_batch.restype = c.c_int
    lib.windq_salient_encode_batch.argtypes = [c.POINTER(windq_salient_item), i32, i32, i64, u32, vp]
    lib.windq_salient_encode_batch.restype = c.c_int
    lib.windq_refine_plan_batch.argtypes = [c.POINTER(windq_refine_item), i32, i32, i64, vp, i32, i32, vp]
    lib.windq_refine_plan_batch.restype = c.c_int
    lib.windq_dequant_plan_batch.argtypes = [c.POINTER(windq_dequant_item), i32, i32, i64, vp]
    lib.windq_dequant_plan_batch.restype = c.c_int
    lib.windq_dequant_gemv.argtypes = [pm, i32, i64, vp, vp, vp, vp, sz, vp, vp, vp, vp, vp, sz, vp]
    lib.windq_dequant_gemv.restype = c.c_int
    lib.windq_dequant_gemv_batch.argtypes = [c.POINTER(windq_gemv_item), i32, i32, i64, vp]
    lib.windq_dequant_gemv_batch.restype = c.c_int
    lib.windq_unit_features_exact_units.argtypes = [vp, i32, i64, i64, i32, i64, c.POINTER(i64)]
    lib.windq_unit_features_exact_units.restype = c.c_int
    lib.windq_status_str.argtypes = [c.c_int]
    lib.windq_status_str.restype = c.c_char_p
    for name in ("windq_calib_stats", "windq_unit_features", "windq_fit_score_all_bits", "windq_plan_layout",
                 "windq_apply_plan", "windq_effective_bits", "windq_salient_select", "windq_salient_encode",
                 "windq_fit_score_all_bits_prot", "windq_apply_plan_prot", "windq_unit_saliency",
                 "windq_heuristic_plan", "windq_fallback_promote", "windq_dequant_plan",
                 "windq_refine_plan", "windq_fit_score_all_bits_batch", "windq_unit_features_batch", "windq_apply_plan_batch", "windq_calib_stats_batch"):
        getattr(lib, name).restype = c.c_int
    _lib = lib
    return lib


def lib():
    return load()


def _check(status: int, where: str):
    if status != WINDQ_OK:
        raise WindqError(status, where)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return WINDQ_F32
    if t.dtype == torch.bfloat16:
        return WINDQ_BF16
    raise WindqError(WINDQ_EDTYPE, "dtype")


def _require_cuda(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise RuntimeError("libwindq runs on the GPU only: pass CUDA tensors (no CPU fallback exists)")


def as_mat(t: torch.Tensor) -> windq_mat:
    assert t.dim() == 2 and t.stride(1) == 1, "row-major 2-D tensor expected"
    return windq_mat(t.data_ptr(), _dtype_code(t), 0, t.shape[0], t.shape[1], t.stride(0))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


def workspace_bytes(call: int, dtype: int, rows: int, cols: int, chunk_w: int = 8, unit_rows: int = 0, K: int = 1) -> int:
    return int(load().windq_workspace_bytes(call, dtype, rows, cols, chunk_w, unit_rows, K))


def _workspace(call, t, chunk_w, unit_rows, K, ws):
    need = workspace_bytes(call, _dtype_code(t), t.shape[0], t.shape[1], chunk_w, unit_rows, K)
    if ws is None:
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=t.device)
    return ws


def n_units(rows: int, cols: int, chunk_w: int, unit_rows: int = 0):
    """(U, rows per unit) of a [rows x cols] matrix."""
    R_u = rows if unit_rows == 0 else unit_rows
    return (rows // R_u) * (cols // chunk_w), R_u


# --------------------------------------------------------------------------- calls
def windq_calib_stats(X: torch.Tensor, want_rms: bool = True, ws: torch.Tensor | None = None,
                      out: torch.Tensor | None = None):
    """-> (s_absmean [C] f32, s_rms [C] f32 or None), device tensors."""
    _require_cuda(X)
    C = X.shape[1]
    s_abs = out if out is not None else torch.empty(C, dtype=torch.float32, device=X.device)
    s_rms = torch.empty(C, dtype=torch.float32, device=X.device) if want_rms else None
    ws = _workspace(CALL_CALIB_STATS, X, 8, 0, 1, ws)
    m = as_mat(X)
    _check(load().windq_calib_stats(ctypes.byref(m), s_abs.data_ptr(), _ptr(s_rms), ws.data_ptr(), ws.numel(),
                                    _stream()), "windq_calib_stats")
    return s_abs, s_rms


def windq_calib_stats_batch(Xs, want_rms: bool = True, wss=None, outs=None):
    """windq_calib_stats for several activation matrices (at most MAX_BATCH) of one element type.
    -> list of (s_absmean, s_rms or None)."""
    n = len(Xs)
    assert (wss is None or len(wss) == n) and (outs is None or len(outs) == n)
    _require_cuda(*Xs)
    mats = [as_mat(X) for X in Xs]
    items = (windq_calib_item * max(n, 1))()
    res, keep = [], []
    for i, X in enumerate(Xs):
        C = X.shape[1]
        s_abs = outs[i] if outs is not None else torch.empty(C, dtype=torch.float32, device=X.device)
        s_rms = torch.empty(C, dtype=torch.float32, device=X.device) if want_rms else None
        ws = _workspace(CALL_CALIB_STATS, X, 8, 0, 1, None if wss is None else wss[i])
        keep.append(ws)
        items[i] = windq_calib_item(ctypes.pointer(mats[i]), s_abs.data_ptr(), _ptr(s_rms), ws.data_ptr(), ws.numel())
        res.append((s_abs, s_rms))
    _check(load().windq_calib_stats_batch(items, n, _stream()), "windq_calib_stats_batch")
    return res


def windq_unit_features(W: torch.Tensor, s: torch.Tensor, chunk_w: int, unit_rows: int = 0,
                        ws: torch.Tensor | None = None, out: torch.Tensor | None = None):
    """-> feat [U x 8] f32 on the device."""
    _require_cuda(W, s)
    U, _ = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
    feat = out if out is not None else torch.empty(U, N_FEAT, dtype=torch.float32, device=W.device)
    ws = _workspace(CALL_UNIT_FEATURES, W, chunk_w, unit_rows, 1, ws)
    m = as_mat(W)
    _check(load().windq_unit_features(ctypes.byref(m), s.data_ptr(), chunk_w, unit_rows, feat.data_ptr(),
                                      ws.data_ptr(), ws.numel(), _stream()), "windq_unit_features")
    return feat


def windq_unit_features_batch(Ws, ss, chunk_w: int, unit_rows: int, wss=None, outs=None):
    """windq_unit_features for several matrices (lists of equal length, at most MAX_BATCH), one launch per pass.
    -> list of feat tensors [U x 8]."""
    n = len(Ws)
    assert len(ss) == n and (wss is None or len(wss) == n) and (outs is None or len(outs) == n)
    _require_cuda(*Ws, *ss)
    mats = [as_mat(W) for W in Ws]
    items = (windq_feat_item * max(n, 1))()
    res, keep = [], []
    for i, (W, s) in enumerate(zip(Ws, ss)):
        U, _ = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
        feat = torch.empty(U, N_FEAT, dtype=torch.float32, device=W.device) if outs is None else outs[i]
        ws = _workspace(CALL_UNIT_FEATURES, W, chunk_w, unit_rows, 1, None if wss is None else wss[i])
        keep.append(ws)
        items[i] = windq_feat_item(ctypes.pointer(mats[i]), s.data_ptr(), feat.data_ptr(), ws.data_ptr(), ws.numel())
        res.append(feat)
    _check(load().windq_unit_features_batch(items, n, chunk_w, unit_rows, _stream()), "windq_unit_features_batch")
    return res


def windq_fit_score_all_bits(W: torch.Tensor, s: torch.Tensor, chunk_w: int, unit_rows: int, clip_grid: torch.Tensor,
                             ws: torch.Tensor | None = None, out=None, mask: torch.Tensor | None = None):
    """clip_grid: host float32 tensor [K].  -> (err [U x 6] f32, clip_idx [U x 4] u8, ref_energy [U] f32).
    With `mask` (device u8 [rows x cols/8]) this is windq_fit_score_all_bits_prot."""
    _require_cuda(W, s, mask)
    assert not clip_grid.is_cuda and clip_grid.dtype == torch.float32 and clip_grid.is_contiguous()
    K = clip_grid.numel()
    U, _ = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
    if out is None:
        err = torch.empty(U, N_ERR, dtype=torch.float32, device=W.device)
        clip_idx = torch.empty(U, 4, dtype=torch.uint8, device=W.device)
        ref = torch.empty(U, dtype=torch.float32, device=W.device)
    else:
        err, clip_idx, ref = out
    ws = _workspace(CALL_FIT_SCORE, W, chunk_w, unit_rows, K, ws)
    m = as_mat(W)
    if mask is None:
        _check(load().windq_fit_score_all_bits(ctypes.byref(m), s.data_ptr(), chunk_w, unit_rows, clip_grid.data_ptr(),
                                               K, err.data_ptr(), clip_idx.data_ptr(), ref.data_ptr(), ws.data_ptr(),
                                               ws.numel(), _stream()), "windq_fit_score_all_bits")
    else:
        _check(load().windq_fit_score_all_bits_prot(ctypes.byref(m), s.data_ptr(), chunk_w, unit_rows, mask.data_ptr(),
                                                    clip_grid.data_ptr(), K, err.data_ptr(), clip_idx.data_ptr(),
                                                    ref.data_ptr(), ws.data_ptr(), ws.numel(), _stream()),
               "windq_fit_score_all_bits_prot")
    return err, clip_idx, ref


def windq_fit_score_all_bits_batch(Ws, ss, chunk_w: int, unit_rows: int, clip_grid: torch.Tensor, wss=None, outs=None,
                                   masks=None):
    """windq_fit_score_all_bits for several matrices (lists of equal length, at most MAX_BATCH) in one launch.
    masks: None, or one protection mask per matrix.  -> list of (err, clip_idx, ref_energy), one per matrix."""
    n = len(Ws)
    assert len(ss) == n and (wss is None or len(wss) == n) and (outs is None or len(outs) == n)
    assert masks is None or len(masks) == n
    _require_cuda(*Ws, *ss, *[m for m in (masks or []) if m is not None])
    assert not clip_grid.is_cuda and clip_grid.dtype == torch.float32 and clip_grid.is_contiguous()
    K = clip_grid.numel()
    mats = [as_mat(W) for W in Ws]
    items = (windq_fit_item * max(n, 1))()
    res, keep = [], []
    for i, (W, s) in enumerate(zip(Ws, ss)):
        U, _ = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
        if outs is None:
            o = (torch.empty(U, N_ERR, dtype=torch.float32, device=W.device),
                 torch.empty(U, 4, dtype=torch.uint8, device=W.device),
                 torch.empty(U, dtype=torch.float32, device=W.device))
        else:
            o = outs[i]
        ws = _workspace(CALL_FIT_SCORE, W, chunk_w, unit_rows, K, None if wss is None else wss[i])
        keep.append(ws)
        items[i] = windq_fit_item(ctypes.pointer(mats[i]), s.data_ptr(), None if masks is None or masks[i] is None else masks[i].data_ptr(),
                                  o[0].data_ptr(), o[1].data_ptr(), o[2].data_ptr(), ws.data_ptr(), ws.numel())
        res.append(o)
    _check(load().windq_fit_score_all_bits_batch(items, n, chunk_w, unit_rows, clip_grid.data_ptr(), K, _stream()),
           "windq_fit_score_all_bits_batch")
    return res


def windq_features_fit_score(W: torch.Tensor, s: torch.Tensor, chunk_w: int, unit_rows: int, clip_grid: torch.Tensor,
                             ws: torch.Tensor | None = None, out=None):
    """Unit features and fit+score from one read of W.  -> (feat [U x 8], err [U x 6], clip_idx [U x 4], ref_energy [U])."""
    _require_cuda(W, s)
    assert not clip_grid.is_cuda and clip_grid.dtype == torch.float32 and clip_grid.is_contiguous()
    K = clip_grid.numel()
    U, _ = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
    if out is None:
        out = (torch.empty(U, N_FEAT, dtype=torch.float32, device=W.device), torch.empty(U, N_ERR, dtype=torch.float32, device=W.device),
               torch.empty(U, 4, dtype=torch.uint8, device=W.device), torch.empty(U, dtype=torch.float32, device=W.device))
    feat, err, clip_idx, ref = out
    ws = _workspace(CALL_FEATURES_FIT_SCORE, W, chunk_w, unit_rows, K, ws)
    m = as_mat(W)
    _check(load().windq_features_fit_score(ctypes.byref(m), s.data_ptr(), chunk_w, unit_rows, clip_grid.data_ptr(), K,
                                           feat.data_ptr(), err.data_ptr(), clip_idx.data_ptr(), ref.data_ptr(),
                                           ws.data_ptr(), ws.numel(), _stream()), "windq_features_fit_score")
    return feat, err, clip_idx, ref


def windq_features_fit_score_batch(Ws, ss, chunk_w: int, unit_rows: int, clip_grid: torch.Tensor, wss=None, outs=None):
    """windq_features_fit_score for several matrices (at most MAX_BATCH) with one launch per kernel.
    -> list of (feat, err, clip_idx, ref_energy)."""
    n = len(Ws)
    assert len(ss) == n and (wss is None or len(wss) == n) and (outs is None or len(outs) == n)
    _require_cuda(*Ws, *ss)
    assert not clip_grid.is_cuda and clip_grid.dtype == torch.float32 and clip_grid.is_contiguous()
    K = clip_grid.numel()
    mats = [as_mat(W) for W in Ws]
    items = (windq_fused_item * max(n, 1))()
    res, keep = [], []
    for i, (W, s) in enumerate(zip(Ws, ss)):
        U, _ = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
        if outs is None:
            o = (torch.empty(U, N_FEAT, dtype=torch.float32, device=W.device), torch.empty(U, N_ERR, dtype=torch.float32, device=W.device),
                 torch.empty(U, 4, dtype=torch.uint8, device=W.device), torch.empty(U, dtype=torch.float32, device=W.device))
        else:
            o = outs[i]
        ws = _workspace(CALL_FEATURES_FIT_SCORE, W, chunk_w, unit_rows, K, None if wss is None else wss[i])
        keep.append(ws)
        items[i] = windq_fused_item(ctypes.pointer(mats[i]), s.data_ptr(), o[0].data_ptr(), o[1].data_ptr(), o[2].data_ptr(),
                                    o[3].data_ptr(), ws.data_ptr(), ws.numel())
        res.append(o)
    _check(load().windq_features_fit_score_batch(items, n, chunk_w, unit_rows, clip_grid.data_ptr(), K, _stream()),
           "windq_features_fit_score_batch")
    return res


def windq_fit_score_all_bits_static(W: torch.Tensor, s: torch.Tensor, chunk_w: int, unit_rows: int, clip_grid: torch.Tensor,
                                    out):
    """windq_fit_score_all_bits on the workspace built into the library: `out` = (err, clip_idx, ref_energy) is
    caller-allocated, nothing is allocated here or in the library."""
    _require_cuda(W, s, *out)
    assert not clip_grid.is_cuda and clip_grid.dtype == torch.float32 and clip_grid.is_contiguous()
    err, clip_idx, ref = out
    m = as_mat(W)
    _check(load().windq_fit_score_all_bits_static(ctypes.byref(m), s.data_ptr(), chunk_w, unit_rows, clip_grid.data_ptr(),
                                                  clip_grid.numel(), err.data_ptr(), clip_idx.data_ptr(), ref.data_ptr(),
                                                  _stream()), "windq_fit_score_all_bits_static")
    return err, clip_idx, ref


def windq_kernel_timer(enable: bool):
    """Switch the event pairs around every main fit+score kernel launch on or off (profiling aid)."""
    _check(load().windq_kernel_timer(1 if enable else 0), "windq_kernel_timer")


def windq_kernel_timer_read():
    """-> (sum of the main fit+score kernel's durations in ms, number of launches) since the last read; waits for the device."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
    _check(load().windq_kernel_timer_read(ctypes.byref(ms), ctypes.byref(n)), "windq_kernel_timer_read")
    return ms.value, n.value


def windq_fit_score_rescored_units(ws: torch.Tensor, W: torch.Tensor, chunk_w: int, unit_rows: int, K: int) -> int:
    """Units of the last fit+score call on workspace `ws` whose 8-bit candidates were scored again on the
    exact route (diagnostic; waits for the device)."""
    _require_cuda(ws)
    n = ctypes.c_int64(0)
    _check(load().windq_fit_score_rescored_units(ws.data_ptr(), _dtype_code(W), W.shape[0], W.shape[1], chunk_w, unit_rows,
                                                 K, ctypes.byref(n)), "windq_fit_score_rescored_units")
    return n.value


def windq_unit_features_exact_units(ws: torch.Tensor, W: torch.Tensor, chunk_w: int, unit_rows: int) -> int:
    """Units of the last unit-features (or fused) call on workspace `ws` that needed the exact pass over
    their weights (diagnostic; waits for the device)."""
    _require_cuda(ws)
    n = ctypes.c_int64(0)
    _check(load().windq_unit_features_exact_units(ws.data_ptr(), _dtype_code(W), W.shape[0], W.shape[1], chunk_w, unit_rows,
                                                  ctypes.byref(n)), "windq_unit_features_exact_units")
    return n.value


def windq_bytes_per_group(action: int, chunk_w: int) -> int:
    return int(load().windq_bytes_per_group(action, chunk_w))


def windq_plan_layout(action: torch.Tensor, rows_per_unit: int, chunk_w: int) -> torch.Tensor:
    """action: host uint8 [U].  -> code_off host int64 [U+1]."""
    assert not action.is_cuda and action.dtype == torch.uint8 and action.is_contiguous()
    U = action.numel()
    off = torch.empty(U + 1, dtype=torch.int64)
    _check(load().windq_plan_layout(action.data_ptr(), U, rows_per_unit, chunk_w, off.data_ptr()), "windq_plan_layout")
    return off


def windq_apply_plan(W: torch.Tensor, chunk_w: int, unit_rows: int, action: torch.Tensor, clip_idx, clip_grid,
                     code_off: torch.Tensor, codes: torch.Tensor | None = None, ws: torch.Tensor | None = None,
                     out=None, mask: torch.Tensor | None = None):
    """action [U] u8, clip_idx [U x 4] u8 or None, code_off [U+1] i64: device tensors; clip_grid host f32 or None.
    -> (codes u8 [code_off[U]], scale f32 [U*R_u], offset f32 [U*R_u]) on the device."""
    _require_cuda(W, action, clip_idx, code_off, codes, mask)
    U, R_u = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
    if codes is None:
        total = int(code_off[-1].item())
        codes = torch.empty(max(total, 16), dtype=torch.uint8, device=W.device)
    if out is None:
        scale = torch.empty(U * R_u, dtype=torch.float32, device=W.device)
        offset = torch.empty(U * R_u, dtype=torch.float32, device=W.device)
    else:
        scale, offset = out
    K = 0 if clip_grid is None else clip_grid.numel()
    ws = _workspace(CALL_APPLY_PLAN, W, chunk_w, unit_rows, 1, ws)
    m = as_mat(W)
    tail = (action.data_ptr(), _ptr(clip_idx), None if clip_grid is None else clip_grid.data_ptr(), K,
            code_off.data_ptr(), codes.data_ptr(), codes.numel(), scale.data_ptr(), offset.data_ptr(),
            ws.data_ptr(), ws.numel(), _stream())
    if mask is None:
        _check(load().windq_apply_plan(ctypes.byref(m), chunk_w, unit_rows, *tail), "windq_apply_plan")
    else:
        _check(load().windq_apply_plan_prot(ctypes.byref(m), chunk_w, unit_rows, mask.data_ptr(), *tail),
               "windq_apply_plan_prot")
    return codes, scale, offset


def windq_apply_plan_batch(Ws, chunk_w: int, unit_rows: int, actions, clip_idxs, clip_grid, code_offs, codes, outs, wss=None,
                           masks=None):
    """windq_apply_plan for several matrices (lists of equal length, at most MAX_BATCH) in one launch.
    actions, clip_idxs (entries may be None), code_offs, codes: device tensors per matrix; outs: (scale, offset) per
    matrix.  clip_grid host f32 or None.  Everything is caller-allocated."""
    n = len(Ws)
    assert all(len(x) == n for x in (actions, clip_idxs, code_offs, codes, outs)) and (wss is None or len(wss) == n)
    _require_cuda(*Ws, *actions, *code_offs, *codes)
    K = 0 if clip_grid is None else clip_grid.numel()
    mats = [as_mat(W) for W in Ws]
    items = (windq_apply_item * max(n, 1))()
    keep = []
    for i, W in enumerate(Ws):
        ws = _workspace(CALL_APPLY_PLAN, W, chunk_w, unit_rows, 1, None if wss is None else wss[i])
        keep.append(ws)
        ci = clip_idxs[i]
        items[i] = windq_apply_item(ctypes.pointer(mats[i]), None if masks is None or masks[i] is None else masks[i].data_ptr(),
                                    actions[i].data_ptr(), None if ci is None else ci.data_ptr(),
                                    code_offs[i].data_ptr(), codes[i].data_ptr(), codes[i].numel(), outs[i][0].data_ptr(),
                                    outs[i][1].data_ptr(), ws.data_ptr(), ws.numel())
    _check(load().windq_apply_plan_batch(items, n, chunk_w, unit_rows, None if clip_grid is None else clip_grid.data_ptr(),
                                         K, _stream()), "windq_apply_plan_batch")
    return [(codes[i], outs[i][0], outs[i][1]) for i in range(n)]


def windq_effective_bits(action: torch.Tensor, n_unit: torch.Tensor, n_prot: torch.Tensor | None = None):
    """Host tensors: action u8 [U], n_unit i64 [U], n_prot i64 [U] or None.  -> (total centibits, total weights)."""
    assert not action.is_cuda and action.dtype == torch.uint8 and n_unit.dtype == torch.int64
    cb, nw = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(load().windq_effective_bits(action.data_ptr(), n_unit.data_ptr(), _ptr(n_prot), action.numel(),
                                       ctypes.byref(cb), ctypes.byref(nw)), "windq_effective_bits")
    return cb.value, nw.value


# ------------------------------------------------------- salient-weight protection
def windq_n_protected(n_unit: int, rate_ppm: int) -> int:
    return int(load().windq_n_protected(n_unit, rate_ppm))


def windq_salient_select(W: torch.Tensor, s: torch.Tensor, chunk_w: int, unit_rows: int, rate_ppm: int,
                         ws: torch.Tensor | None = None, out: torch.Tensor | None = None):
    """-> mask u8 [rows x cols/8] on the device: bit (c mod 8) of byte c/8 set where weight (row, c) is protected."""
    _require_cuda(W, s)
    mask = out if out is not None else torch.empty(W.shape[0], W.shape[1] // 8, dtype=torch.uint8, device=W.device)
    ws = _workspace(CALL_SALIENT, W, chunk_w, unit_rows, 1, ws)
    m = as_mat(W)
    _check(load().windq_salient_select(ctypes.byref(m), s.data_ptr(), chunk_w, unit_rows, rate_ppm, mask.data_ptr(),
                                       ws.data_ptr(), ws.numel(), _stream()), "windq_salient_select")
    return mask


def windq_salient_encode(W: torch.Tensor, s: torch.Tensor, chunk_w: int, unit_rows: int, mask: torch.Tensor,
                         rate_ppm: int, ws: torch.Tensor | None = None, out=None):
    """-> (prot_codes i8 [U x n_p], prot_scale f32 [U], err_prot f32 [U]) on the device."""
    _require_cuda(W, s, mask)
    U, R_u = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
    n_p = windq_n_protected(R_u * chunk_w, rate_ppm)
    if out is None:
        codes = torch.empty(U, max(n_p, 1), dtype=torch.int8, device=W.device)[:, :n_p]
        codes = torch.empty(U, n_p, dtype=torch.int8, device=W.device) if n_p > 0 else codes
        scale = torch.empty(U, dtype=torch.float32, device=W.device)
        err = torch.empty(U, dtype=torch.float32, device=W.device)
    else:
        codes, scale, err = out
    ws = _workspace(CALL_SALIENT, W, chunk_w, unit_rows, 1, ws)
    m = as_mat(W)
    _check(load().windq_salient_encode(ctypes.byref(m), s.data_ptr(), chunk_w, unit_rows, mask.data_ptr(), rate_ppm,
                                       codes.data_ptr() if n_p > 0 else None, scale.data_ptr(), err.data_ptr(),
                                       ws.data_ptr(), ws.numel(), _stream()), "windq_salient_encode")
    return codes, scale, err


def _salient_outs(W, chunk_w, unit_rows, rate_ppm):
    U, R_u = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
    n_p = windq_n_protected(R_u * chunk_w, rate_ppm)
    return (torch.empty(U, n_p, dtype=torch.int8, device=W.device), torch.empty(U, dtype=torch.float32, device=W.device),
            torch.empty(U, dtype=torch.float32, device=W.device))


def windq_salient_select_batch(Ws, ss, chunk_w: int, unit_rows: int, rate_ppm: int, wss=None, outs=None):
    """windq_salient_select for several matrices (lists of equal length, at most MAX_BATCH): one launch per kernel.
    -> [mask u8 [rows x cols/8]] per matrix."""
    n = len(Ws)
    assert len(ss) == n and (wss is None or len(wss) == n) and (outs is None or len(outs) == n)
    _require_cuda(*Ws, *ss)
    mats = [as_mat(W) for W in Ws]
    items = (windq_salient_item * max(n, 1))()
    masks, keep = [], []
    for i, W in enumerate(Ws):
        mask = outs[i] if outs is not None else torch.empty(W.shape[0], W.shape[1] // 8, dtype=torch.uint8, device=W.device)
        ws = _workspace(CALL_SALIENT, W, chunk_w, unit_rows, 1, None if wss is None else wss[i])
        masks.append(mask)
        keep.append(ws)
        items[i] = windq_salient_item(ctypes.pointer(mats[i]), ss[i].data_ptr(), mask.data_ptr(), None, None, None,
                                      ws.data_ptr(), ws.numel())
    _check(load().windq_salient_select_batch(items, n, chunk_w, unit_rows, rate_ppm, _stream()), "windq_salient_select_batch")
    return masks


def windq_salient_encode_batch(Ws, ss, chunk_w: int, unit_rows: int, masks, rate_ppm: int, wss=None, outs=None):
    """windq_salient_encode for several matrices: one launch per kernel.
    -> [(prot_codes i8 [U x n_p], prot_scale f32 [U], err_prot f32 [U])] per matrix."""
    n = len(Ws)
    assert len(ss) == n and len(masks) == n and (wss is None or len(wss) == n) and (outs is None or len(outs) == n)
    _require_cuda(*Ws, *ss, *masks)
    mats = [as_mat(W) for W in Ws]
    items = (windq_salient_item * max(n, 1))()
    res, keep = [], []
    for i, W in enumerate(Ws):
        codes, scale, err = outs[i] if outs is not None else _salient_outs(W, chunk_w, unit_rows, rate_ppm)
        ws = _workspace(CALL_SALIENT, W, chunk_w, unit_rows, 1, None if wss is None else wss[i])
        res.append((codes, scale, err))
        keep.append(ws)
        items[i] = windq_salient_item(ctypes.pointer(mats[i]), ss[i].data_ptr(), masks[i].data_ptr(),
                                      codes.data_ptr() if codes.numel() > 0 else None, scale.data_ptr(), err.data_ptr(),
                                      ws.data_ptr(), ws.numel())
    _check(load().windq_salient_encode_batch(items, n, chunk_w, unit_rows, rate_ppm, _stream()), "windq_salient_encode_batch")
    return res


# --------------------------------------------- heuristic allocator and fallback
def windq_unit_saliency(W: torch.Tensor, s: torch.Tensor, chunk_w: int, unit_rows: int = 0,
                        ws: torch.Tensor | None = None, out: torch.Tensor | None = None):
    """-> sal f32 [U] on the device: mean of |w| * |s_c| over each unit."""
    _require_cuda(W, s)
    U, _ = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
    sal = out if out is not None else torch.empty(U, dtype=torch.float32, device=W.device)
    ws = _workspace(CALL_UNIT_SALIENCY, W, chunk_w, unit_rows, 1, ws)
    m = as_mat(W)
    _check(load().windq_unit_saliency(ctypes.byref(m), s.data_ptr(), chunk_w, unit_rows, sal.data_ptr(), ws.data_ptr(),
                                      ws.numel(), _stream()), "windq_unit_saliency")
    return sal


def windq_heuristic_plan(sal: torch.Tensor, n_unit: torch.Tensor, n_prot: torch.Tensor | None, target_centibits: int,
                         frac_1bit_ppm: int = 0, frac_ternary_ppm: int = 0):
    """Host tensors: sal f32 [U], n_unit i64 [U], n_prot i64 [U] or None.  -> (action u8 [U], total centibits, feasible)."""
    assert not sal.is_cuda and sal.dtype == torch.float32 and sal.is_contiguous() and n_unit.dtype == torch.int64
    U = sal.numel()
    action = torch.empty(U, dtype=torch.uint8)
    cb, ok = ctypes.c_int64(0), ctypes.c_int32(0)
    _check(load().windq_heuristic_plan(sal.data_ptr(), n_unit.data_ptr(), _ptr(n_prot), U, target_centibits,
                                       frac_1bit_ppm, frac_ternary_ppm, action.data_ptr(), ctypes.byref(cb),
                                       ctypes.byref(ok)), "windq_heuristic_plan")
    return action, cb.value, bool(ok.value)


def windq_fallback_promote(action: torch.Tensor, err: torch.Tensor, ref: torch.Tensor, max_rel_err: float):
    """Host tensors: action u8 [U] (updated in place), err f32 [U x 6], ref f32 [U].  -> number of units changed."""
    assert not action.is_cuda and action.dtype == torch.uint8 and not err.is_cuda and err.dtype == torch.float32
    assert err.is_contiguous() and not ref.is_cuda and ref.dtype == torch.float32
    n = ctypes.c_int64(0)
    _check(load().windq_fallback_promote(action.data_ptr(), err.data_ptr(), ref.data_ptr(), action.numel(),
                                         max_rel_err, ctypes.byref(n)), "windq_fallback_promote")
    return n.value


# ------------------------------------------------------------------- dequantisation
def windq_dequant_plan(W: torch.Tensor, s: torch.Tensor, chunk_w: int, unit_rows: int, action: torch.Tensor,
                       code_off: torch.Tensor, codes: torch.Tensor, scale: torch.Tensor, offset: torch.Tensor,
                       mask: torch.Tensor | None = None, want_w_hat: bool = True, ws: torch.Tensor | None = None):
    """Device tensors as windq_apply_plan wrote them.  -> (err f32 [U], w_hat f32 [rows x cols] or None)."""
    _require_cuda(W, s, action, code_off, codes, scale, offset, mask)
    U, _ = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
    err = torch.empty(U, dtype=torch.float32, device=W.device)
    w_hat = torch.empty(W.shape[0], W.shape[1], dtype=torch.float32, device=W.device) if want_w_hat else None
    ws = _workspace(CALL_DEQUANT, W, chunk_w, unit_rows, 1, ws)
    m = as_mat(W)
    _check(load().windq_dequant_plan(ctypes.byref(m), s.data_ptr(), chunk_w, unit_rows, _ptr(mask), action.data_ptr(),
                                     code_off.data_ptr(), codes.data_ptr(), codes.numel(), scale.data_ptr(),
                                     offset.data_ptr(), err.data_ptr(), _ptr(w_hat), ws.data_ptr(), ws.numel(),
                                     _stream()), "windq_dequant_plan")
    return err, w_hat


# ------------------------------------------------------------- iterative refinement
def windq_refine_plan(W: torch.Tensor, s: torch.Tensor, chunk_w: int, unit_rows: int, action: torch.Tensor, clip_idx,
                      clip_grid, code_off: torch.Tensor, n_iter: int, codes: torch.Tensor | None = None,
                      mask: torch.Tensor | None = None, ws: torch.Tensor | None = None):
    """windq_apply_plan with n_iter rounds of closed-form scale refinement.
    -> (codes u8, scale f32 [U*R_u], offset f32 [U*R_u], err f32 [U]) on the device."""
    _require_cuda(W, s, action, clip_idx, code_off, codes, mask)
    U, R_u = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
    if codes is None:
        codes = torch.empty(max(int(code_off[-1].item()), 16), dtype=torch.uint8, device=W.device)
    scale = torch.empty(U * R_u, dtype=torch.float32, device=W.device)
    offset = torch.empty(U * R_u, dtype=torch.float32, device=W.device)
    err = torch.empty(U, dtype=torch.float32, device=W.device)
    K = 0 if clip_grid is None else clip_grid.numel()
    ws = _workspace(CALL_REFINE, W, chunk_w, unit_rows, 1, ws)
    m = as_mat(W)
    _check(load().windq_refine_plan(ctypes.byref(m), s.data_ptr(), chunk_w, unit_rows, _ptr(mask), action.data_ptr(),
                                    _ptr(clip_idx), None if clip_grid is None else clip_grid.data_ptr(), K, n_iter,
                                    code_off.data_ptr(), codes.data_ptr(), codes.numel(), scale.data_ptr(),
                                    offset.data_ptr(), err.data_ptr(), ws.data_ptr(), ws.numel(), _stream()),
           "windq_refine_plan")
    return codes, scale, offset, err


def windq_refine_plan_batch(Ws, ss, chunk_w: int, unit_rows: int, actions, clip_idxs, clip_grid, code_offs, n_iter: int,
                            codes, outs=None, masks=None, wss=None):
    """windq_refine_plan for several matrices (lists of equal length, at most MAX_BATCH) in one launch.
    clip_idxs and masks: lists whose entries may be None (masks itself may be None); codes: caller-allocated u8
    tensors; outs: (scale, offset, err) per matrix or None.  -> [(codes, scale, offset, err)] per matrix."""
    n = len(Ws)
    assert all(len(x) == n for x in (ss, actions, clip_idxs, code_offs, codes))
    _require_cuda(*Ws, *ss, *actions, *code_offs, *codes)
    K = 0 if clip_grid is None else clip_grid.numel()
    mats = [as_mat(W) for W in Ws]
    items = (windq_refine_item * max(n, 1))()
    res, keep = [], []
    for i, W in enumerate(Ws):
        U, R_u = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
        if outs is not None:
            scale, offset, err = outs[i]
        else:
            scale = torch.empty(U * R_u, dtype=torch.float32, device=W.device)
            offset = torch.empty(U * R_u, dtype=torch.float32, device=W.device)
            err = torch.empty(U, dtype=torch.float32, device=W.device)
        ws = _workspace(CALL_REFINE, W, chunk_w, unit_rows, 1, None if wss is None else wss[i])
        keep.append(ws)
        res.append((codes[i], scale, offset, err))
        items[i] = windq_refine_item(ctypes.pointer(mats[i]), ss[i].data_ptr(), None if masks is None else _ptr(masks[i]),
                                     actions[i].data_ptr(), _ptr(clip_idxs[i]), code_offs[i].data_ptr(),
                                     codes[i].data_ptr(), codes[i].numel(), scale.data_ptr(), offset.data_ptr(),
                                     err.data_ptr(), ws.data_ptr(), ws.numel())
    _check(load().windq_refine_plan_batch(items, n, chunk_w, unit_rows, None if clip_grid is None else clip_grid.data_ptr(),
                                          K, n_iter, _stream()), "windq_refine_plan_batch")
    return res


def windq_dequant_plan_batch(Ws, ss, chunk_w: int, unit_rows: int, actions, code_offs, codes, scales, offsets, masks=None,
                             want_w_hat: bool = True, wss=None, outs=None):
    """windq_dequant_plan for several matrices (lists of equal length, at most MAX_BATCH) in one launch.
    outs: (err, w_hat or None) per matrix, or None to allocate.  -> [(err f32 [U], w_hat f32 [rows x cols] or None)]."""
    n = len(Ws)
    assert all(len(x) == n for x in (ss, actions, code_offs, codes, scales, offsets))
    _require_cuda(*Ws, *ss, *actions, *code_offs, *codes, *scales, *offsets)
    mats = [as_mat(W) for W in Ws]
    items = (windq_dequant_item * max(n, 1))()
    res, keep = [], []
    for i, W in enumerate(Ws):
        U, _ = n_units(W.shape[0], W.shape[1], chunk_w, unit_rows)
        if outs is not None:
            err, w_hat = outs[i]
        else:
            err = torch.empty(U, dtype=torch.float32, device=W.device)
            w_hat = torch.empty(W.shape[0], W.shape[1], dtype=torch.float32, device=W.device) if want_w_hat else None
        ws = _workspace(CALL_DEQUANT, W, chunk_w, unit_rows, 1, None if wss is None else wss[i])
        keep.append(ws)
        res.append((err, w_hat))
        items[i] = windq_dequant_item(ctypes.pointer(mats[i]), ss[i].data_ptr(), None if masks is None else _ptr(masks[i]),
                                      actions[i].data_ptr(), code_offs[i].data_ptr(), codes[i].data_ptr(), codes[i].numel(),
                                      scales[i].data_ptr(), offsets[i].data_ptr(), _ptr(err), _ptr(w_hat), ws.data_ptr(),
                                      ws.numel())
    _check(load().windq_dequant_plan_batch(items, n, chunk_w, unit_rows, _stream()), "windq_dequant_plan_batch")
    return res


def windq_dequant_gemv(W: torch.Tensor, chunk_w: int, unit_rows: int, action: torch.Tensor, code_off: torch.Tensor,
                       codes: torch.Tensor, scale: torch.Tensor, offset: torch.Tensor, x: torch.Tensor,
                       mask: torch.Tensor | None = None, ws: torch.Tensor | None = None, out: torch.Tensor | None = None):
    """y = W_hat x from the packed plan (device tensors as windq_apply_plan wrote them; x f32 [cols]).  -> y f32 [rows]."""
    _require_cuda(W, action, code_off, codes, scale, offset, x, mask)
    assert x.dtype == torch.float32 and x.is_contiguous()
    y = out if out is not None else torch.empty(W.shape[0], dtype=torch.float32, device=W.device)
    ws = _workspace(CALL_DEQUANT_GEMV, W, chunk_w, unit_rows, 1, ws)
    m = as_mat(W)
    _check(load().windq_dequant_gemv(ctypes.byref(m), chunk_w, unit_rows, _ptr(mask), action.data_ptr(), code_off.data_ptr(),
                                     codes.data_ptr(), codes.numel(), scale.data_ptr(), offset.data_ptr(), x.data_ptr(),
                                     y.data_ptr(), ws.data_ptr(), ws.numel(), _stream()), "windq_dequant_gemv")
    return y


def windq_dequant_gemv_batch(Ws, chunk_w: int, unit_rows: int, actions, code_offs, codes, scales, offsets, xs, masks=None,
                             wss=None, outs=None):
    """windq_dequant_gemv for several matrices (lists of equal length, at most MAX_BATCH) in one launch.  -> [y]."""
    n = len(Ws)
    assert all(len(v) == n for v in (actions, code_offs, codes, scales, offsets, xs))
    _require_cuda(*Ws, *actions, *code_offs, *codes, *scales, *offsets, *xs)
    mats = [as_mat(W) for W in Ws]
    items = (windq_gemv_item * max(n, 1))()
    ys, keep = [], []
    for i, W in enumerate(Ws):
        assert xs[i].dtype == torch.float32 and xs[i].is_contiguous()
        y = outs[i] if outs is not None else torch.empty(W.shape[0], dtype=torch.float32, device=W.device)
        ws = _workspace(CALL_DEQUANT_GEMV, W, chunk_w, unit_rows, 1, None if wss is None else wss[i])
        ys.append(y)
        keep.append(ws)
        items[i] = windq_gemv_item(ctypes.pointer(mats[i]), None if masks is None else _ptr(masks[i]), actions[i].data_ptr(),
                                   code_offs[i].data_ptr(), codes[i].data_ptr(), codes[i].numel(), scales[i].data_ptr(),
                                   offsets[i].data_ptr(), xs[i].data_ptr(), y.data_ptr(), ws.data_ptr(), ws.numel())
    _check(load().windq_dequant_gemv_batch(items, n, chunk_w, unit_rows, _stream()), "windq_dequant_gemv_batch")
    return ys
