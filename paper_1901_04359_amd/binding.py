"""Thin ctypes binding over libgtopk.so (argument marshalling only).

Every function has the name and argument order of its C entry point in
include/gtopk.h, takes torch CUDA(ROCm) tensors where the C side takes device
pointers, checks dtypes/devices/contiguity, passes raw pointers and the current
stream, and raises `GtopkError` on a non-zero status.  No step of the method
runs in Python and there is no fallback: if the library is missing, loading
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libgtopk.so")
_lib: Optional[ctypes.CDLL] = None

EXPORTS = (
    "gtopk_status_string", "gtopk_workspace_bytes", "gtopk_merge_workspace_bytes",
    "gtopk_local_select", "gtopk_merge", "gtopk_tree", "gtopk_residual_restore", "gtopk_step",
    "gtopk_step_static", "gtopk_step_carry",
    "gtopk_apply_update", "gtopk_dense_mask",
    "gtopk_allreduce_workspace_bytes", "gtopk_topk_allreduce", "gtopk_dense_topk",
    "gtopk_step_timed", "gtopk_probe_stream", "gtopk_debug_candidate_counts", "gtopk_debug_plan",
    "gtopk_debug_merge_kept",
)

GTOPK_OK, GTOPK_EINVAL, GTOPK_EWORKSPACE, GTOPK_EALIGN, GTOPK_EHIP = 0, -1, -2, -3, -4


class GtopkError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Load libgtopk.so (built by `python -m paper_1901_04359_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_1901_04359_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(_LIB_PATH)
    c = ctypes
    vp, i32, i64, sz = c.c_void_p, c.c_int32, c.c_int64, c.c_size_t
    lib.gtopk_status_string.restype = c.c_char_p
    lib.gtopk_status_string.argtypes = [c.c_int]
    lib.gtopk_workspace_bytes.restype = sz
    lib.gtopk_workspace_bytes.argtypes = [i64, i32, i32]
    lib.gtopk_merge_workspace_bytes.restype = sz
    lib.gtopk_merge_workspace_bytes.argtypes = [i32, i32]
    lib.gtopk_local_select.restype = c.c_int
    lib.gtopk_local_select.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp, vp, sz, vp]
    lib.gtopk_merge.restype = c.c_int
    lib.gtopk_merge.argtypes = [vp, vp, vp, vp, i32, i32, i64, vp, vp, i64, vp, sz, vp]
    lib.gtopk_tree.restype = c.c_int
    lib.gtopk_tree.argtypes = [vp, vp, i32, i32, vp, vp, vp, sz, vp]
    lib.gtopk_residual_restore.restype = c.c_int
    lib.gtopk_residual_restore.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp]
    lib.gtopk_step.restype = c.c_int
    lib.gtopk_step.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.gtopk_step_static.restype = c.c_int
    lib.gtopk_step_static.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp, vp, vp, vp]
    lib.gtopk_apply_update.restype = c.c_int
    lib.gtopk_apply_update.argtypes = [vp, i64, i64, i32, i32, vp, vp, c.c_float, vp]
    lib.gtopk_dense_mask.restype = c.c_int
    lib.gtopk_dense_mask.argtypes = [vp, i32, i64, vp, vp]
    lib.gtopk_allreduce_workspace_bytes.restype = sz
    lib.gtopk_allreduce_workspace_bytes.argtypes = [i64, i32]
    lib.gtopk_topk_allreduce.restype = c.c_int
    lib.gtopk_topk_allreduce.argtypes = [vp, vp, i32, i32, i64, vp, vp, sz, vp]
    lib.gtopk_dense_topk.restype = c.c_int
    lib.gtopk_dense_topk.argtypes = [vp, i64, i32, vp, vp, vp, sz, vp]
    lib.gtopk_step_timed.restype = c.c_int
    lib.gtopk_step_timed.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp,
                                     c.POINTER(c.c_void_p)]
    lib.gtopk_step_carry.restype = c.c_int
    lib.gtopk_step_carry.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.gtopk_probe_stream.restype = c.c_int
    lib.gtopk_probe_stream.argtypes = [vp, vp, i64, i32, vp, vp]
    lib.gtopk_debug_plan.restype = c.c_int
    lib.gtopk_debug_plan.argtypes = [i64, i32, i32, c.POINTER(c.c_uint32)]
    lib.gtopk_debug_merge_kept.restype = c.c_int
    lib.gtopk_debug_merge_kept.argtypes = [vp, i32, i32, c.POINTER(c.c_uint32)]
    lib.gtopk_debug_candidate_counts.restype = c.c_int
    lib.gtopk_debug_candidate_counts.argtypes = [vp, i64, i32, i32, c.POINTER(c.c_uint32),
                                                 c.POINTER(c.c_uint32)]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().gtopk_status_string(int(status)).decode()


def gtopk_workspace_bytes(m: int, k: int, P: int) -> int:
    return int(load().gtopk_workspace_bytes(m, k, P))


def gtopk_merge_workspace_bytes(k: int, batch: int) -> int:
    return int(load().gtopk_merge_workspace_bytes(k, batch))


# -- marshalling helpers ------------------------------------------------------

def _torch():
    import torch
    return torch


def _ptr(t, dtype, name: str, allow_none: bool = False):
    if t is None:
        if allow_none:
            return None
        raise TypeError(f"{name} is None")
    torch = _torch()
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    torch = _torch()
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _rows(t, name: str):
    """(m, stride) of a [P][m] tensor whose rows are contiguous."""
    if t.dim() != 2 or t.stride(1) != 1:
        raise ValueError(f"{name} must be 2-D with contiguous rows")
    return t.shape[1], (t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1]))


def _check(status: int, where: str):
    if status != 0:
        raise GtopkError(status, where)


def alloc_workspace(m: int, k: int, P: int, device="cuda"):
    torch = _torch()
    n = gtopk_workspace_bytes(m, k, P)
    if n == 0:
        raise GtopkError(GTOPK_EINVAL, "gtopk_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def alloc_merge_workspace(k: int, batch: int, device="cuda"):
    torch = _torch()
    n = gtopk_merge_workspace_bytes(k, batch)
    if n == 0:
        raise GtopkError(GTOPK_EINVAL, "gtopk_merge_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


# -- entry points -------------------------------------------------------------
# index tensors are torch.int32 holding the uint32 bit patterns

def gtopk_local_select(grad, residual, k: int, out_idx, out_val, ws) -> None:
    torch = _torch()
    m, stride = _rows(residual, "residual")
    mg, sg = _rows(grad, "grad")
    P = residual.shape[0]
    if (mg, grad.shape[0]) != (m, P) or (P > 1 and sg != stride):
        raise ValueError("grad and residual must have the same shape and row stride")
    rc = load().gtopk_local_select(
        _ptr(grad, torch.float32, "grad"), _ptr(residual, torch.float32, "residual"),
        m, stride, P, k, _ptr(out_idx, torch.int32, "out_idx"),
        _ptr(out_val, torch.float32, "out_val"), _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream())
    _check(rc, "gtopk_local_select")


def gtopk_merge(a_idx, a_val, b_idx, b_val, k: int, batch: int, in_stride: int,
                out_idx, out_val, out_stride: int, ws) -> None:
    torch = _torch()
    rc = load().gtopk_merge(
        _ptr(a_idx, torch.int32, "a_idx"), _ptr(a_val, torch.float32, "a_val"),
        _ptr(b_idx, torch.int32, "b_idx"), _ptr(b_val, torch.float32, "b_val"),
        k, batch, in_stride, _ptr(out_idx, torch.int32, "out_idx"),
        _ptr(out_val, torch.float32, "out_val"), out_stride,
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream())
    _check(rc, "gtopk_merge")


def gtopk_tree(loc_idx, loc_val, P: int, k: int, g_idx, g_val, ws) -> None:
    torch = _torch()
    rc = load().gtopk_tree(
        _ptr(loc_idx, torch.int32, "loc_idx"), _ptr(loc_val, torch.float32, "loc_val"), P, k,
        _ptr(g_idx, torch.int32, "g_idx"), _ptr(g_val, torch.float32, "g_val"),
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream())
    _check(rc, "gtopk_tree")


def gtopk_residual_restore(residual, k: int, loc_idx, loc_val, g_idx) -> None:
    torch = _torch()
    m, stride = _rows(residual, "residual")
    P = residual.shape[0]
    rc = load().gtopk_residual_restore(
        _ptr(residual, torch.float32, "residual"), m, stride, P, k,
        _ptr(loc_idx, torch.int32, "loc_idx"), _ptr(loc_val, torch.float32, "loc_val"),
        _ptr(g_idx, torch.int32, "g_idx"), _stream())
    _check(rc, "gtopk_residual_restore")


def gtopk_step(grad, residual, k: int, g_idx, g_val, loc_idx, loc_val, ws) -> None:
    torch = _torch()
    m, stride = _rows(residual, "residual")
    mg, sg = _rows(grad, "grad")
    P = residual.shape[0]
    if (mg, grad.shape[0]) != (m, P) or (P > 1 and sg != stride):
        raise ValueError("grad and residual must have the same shape and row stride")
    rc = load().gtopk_step(
        _ptr(grad, torch.float32, "grad"), _ptr(residual, torch.float32, "residual"),
        m, stride, P, k, _ptr(g_idx, torch.int32, "g_idx"), _ptr(g_val, torch.float32, "g_val"),
        _ptr(loc_idx, torch.int32, "loc_idx", allow_none=True),
        _ptr(loc_val, torch.float32, "loc_val", allow_none=True),
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream())
    _check(rc, "gtopk_step")


STATIC_WORKSPACE_BYTES = 16 << 20


def gtopk_step_static(grad, residual, k: int, g_idx, g_val, loc_idx, loc_val) -> None:
    """gtopk_step on the library's own static workspace (no allocation anywhere)."""
    torch = _torch()
    m, stride = _rows(residual, "residual")
    mg, sg = _rows(grad, "grad")
    P = residual.shape[0]
    if (mg, grad.shape[0]) != (m, P) or (P > 1 and sg != stride):
        raise ValueError("grad and residual must have the same shape and row stride")
    rc = load().gtopk_step_static(
        _ptr(grad, torch.float32, "grad"), _ptr(residual, torch.float32, "residual"),
        m, stride, P, k, _ptr(g_idx, torch.int32, "g_idx"), _ptr(g_val, torch.float32, "g_val"),
        _ptr(loc_idx, torch.int32, "loc_idx", allow_none=True),
        _ptr(loc_val, torch.float32, "loc_val", allow_none=True), _stream())
    _check(rc, "gtopk_step_static")


def gtopk_apply_update(weights, k: int, g_idx, g_val, lr: float) -> None:
    """weights: [copies][m] (rows contiguous) or [m]."""
    torch = _torch()
    w2 = weights if weights.dim() == 2 else weights.view(1, -1)
    m, stride = _rows(w2, "weights")
    rc = load().gtopk_apply_update(
        _ptr(w2, torch.float32, "weights"), m, stride, w2.shape[0], k,
        _ptr(g_idx, torch.int32, "g_idx"), _ptr(g_val, torch.float32, "g_val"),
        ctypes.c_float(lr), _stream())
    _check(rc, "gtopk_apply_update")


def gtopk_dense_mask(g_idx, k: int, mask) -> None:
    torch = _torch()
    rc = load().gtopk_dense_mask(_ptr(g_idx, torch.int32, "g_idx"), k, mask.numel(),
                                 _ptr(mask, torch.uint8, "mask"), _stream())
    _check(rc, "gtopk_dense_mask")


def gtopk_allreduce_workspace_bytes(m: int, P: int) -> int:
    return int(load().gtopk_allreduce_workspace_bytes(m, P))


def alloc_allreduce_workspace(m: int, P: int, device="cuda"):
    torch = _torch()
    n = gtopk_allreduce_workspace_bytes(m, P)
    if n == 0:
        raise GtopkError(GTOPK_EINVAL, "gtopk_allreduce_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def gtopk_topk_allreduce(loc_idx, loc_val, P: int, k: int, dense, ws) -> None:
    """loc_idx / loc_val: [P][k] contiguous; dense: [m] float32 (output)."""
    torch = _torch()
    rc = load().gtopk_topk_allreduce(
        _ptr(loc_idx, torch.int32, "loc_idx"), _ptr(loc_val, torch.float32, "loc_val"), P, k,
        dense.numel(), _ptr(dense, torch.float32, "dense"), _ptr(ws, torch.uint8, "ws"),
        ws.numel(), _stream())
    _check(rc, "gtopk_topk_allreduce")


def gtopk_dense_topk(dense, k: int, g_idx, g_val, ws) -> None:
    """dense: [m] float32; ws from alloc_workspace(m, k, 1)."""
    torch = _torch()
    rc = load().gtopk_dense_topk(
        _ptr(dense, torch.float32, "dense"), dense.numel(), k,
        _ptr(g_idx, torch.int32, "g_idx"), _ptr(g_val, torch.float32, "g_val"),
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream())
    _check(rc, "gtopk_dense_topk")


def gtopk_step_carry(grad, residual, k: int, g_idx, g_val, loc_idx, loc_val, thr_state, ws) -> None:
    """gtopk_step with the speculative thresholds carried in `thr_state` ([P][4] int32, zeroed
    by the caller before the first call)."""
    torch = _torch()
    m, stride = _rows(residual, "residual")
    mg, sg = _rows(grad, "grad")
    P = residual.shape[0]
    if (mg, grad.shape[0]) != (m, P) or (P > 1 and sg != stride):
        raise ValueError("grad and residual must have the same shape and row stride")
    if thr_state.numel() != 4 * P:
        raise ValueError("thr_state must hold 4 words per worker")
    rc = load().gtopk_step_carry(
        _ptr(grad, torch.float32, "grad"), _ptr(residual, torch.float32, "residual"),
        m, stride, P, k, _ptr(g_idx, torch.int32, "g_idx"), _ptr(g_val, torch.float32, "g_val"),
        _ptr(loc_idx, torch.int32, "loc_idx", allow_none=True),
        _ptr(loc_val, torch.float32, "loc_val", allow_none=True),
        _ptr(thr_state, torch.int32, "thr_state"),
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream())
    _check(rc, "gtopk_step_carry")


def gtopk_step_timed(grad, residual, k: int, g_idx, g_val, loc_idx, loc_val, ws, events,
                     thr_state=None) -> None:
    """gtopk_step (or, with thr_state, gtopk_step_carry) that records the caller's six raw
    hipEvent_t handles (ints) at its stage boundaries."""
    torch = _torch()
    m, stride = _rows(residual, "residual")
    mg, sg = _rows(grad, "grad")
    P = residual.shape[0]
    if (mg, grad.shape[0]) != (m, P) or (P > 1 and sg != stride):
        raise ValueError("grad and residual must have the same shape and row stride")
    if len(events) != 6:
        raise ValueError("six event handles are needed")
    arr = (ctypes.c_void_p * 6)(*events)
    rc = load().gtopk_step_timed(
        _ptr(grad, torch.float32, "grad"), _ptr(residual, torch.float32, "residual"),
        m, stride, P, k, _ptr(g_idx, torch.int32, "g_idx"), _ptr(g_val, torch.float32, "g_val"),
        _ptr(loc_idx, torch.int32, "loc_idx", allow_none=True),
        _ptr(loc_val, torch.float32, "loc_val", allow_none=True),
        _ptr(thr_state, torch.int32, "thr_state", allow_none=True),
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream(), arr)
    _check(rc, "gtopk_step_timed")


def gtopk_probe_stream(a, b, n: int, mode: int, sink=None) -> None:
    """a, b: float32 GPU tensors of at least n elements (b is updated in mode 0)."""
    torch = _torch()
    rc = load().gtopk_probe_stream(
        _ptr(a, torch.float32, "a"), _ptr(b, torch.float32, "b"), n, mode,
        _ptr(sink, torch.float32, "sink", allow_none=True), _stream())
    _check(rc, "gtopk_probe_stream")


PLAN_FIELDS = ("tile_stride", "n_tiles", "tile_len", "target", "capacity", "pass_histogram",
               "small_path", "run_groups", "small_tile_stride", "small_n_tiles", "small_target",
               "merge_filtered", "merge_tile_stride", "merge_n_tiles", "merge_target", "reserved")


def gtopk_debug_plan(m: int, k: int, P: int) -> dict:
    """Layout of the local selection for these sizes (host only; see gtopk.h)."""
    plan = (ctypes.c_uint32 * len(PLAN_FIELDS))()
    _check(load().gtopk_debug_plan(m, k, P, plan), "gtopk_debug_plan")
    return dict(zip(PLAN_FIELDS, (int(x) for x in plan)))


def gtopk_debug_merge_kept(ws, k: int, batch: int):
    """Slots of each pair's union that reached its speculative threshold in the last completed
    gtopk_merge on `ws` (large k only; see gtopk.h)."""
    torch = _torch()
    torch.cuda.synchronize()
    kept = (ctypes.c_uint32 * batch)()
    _check(load().gtopk_debug_merge_kept(_ptr(ws, torch.uint8, "ws"), k, batch, kept), "gtopk_debug_merge_kept")
    return list(kept)


def gtopk_debug_candidate_counts(ws, m: int, k: int, P: int):
    """(per-worker candidate counts, list capacity) of the last completed select on `ws`."""
    torch = _torch()
    torch.cuda.synchronize()
    counts = (ctypes.c_uint32 * P)()
    cap = ctypes.c_uint32(0)
    rc = load().gtopk_debug_candidate_counts(_ptr(ws, torch.uint8, "ws"), m, k, P, counts,
                                             ctypes.byref(cap))
    _check(rc, "gtopk_debug_candidate_counts")
    return list(counts), int(cap.value)
