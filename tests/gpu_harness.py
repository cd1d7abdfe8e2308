"""Helpers for the GPU parity tests: move numpy arrays to the device, call the
library through the ctypes binding (the C ABI), bring results back as numpy."""
import os
import sys
import time

import numpy as np

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_CASE_LOG = os.path.join(_ROOT, "gpurun_out", "gpu_cases.log")


def say(msg: str) -> None:
    """Name the case before the GPU step runs, and flush, so a dead box names its test.
    The line also goes to a log file that a test runner's output capture does not hold back."""
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()
    try:
        os.makedirs(os.path.dirname(_CASE_LOG), exist_ok=True)
        with open(_CASE_LOG, "a") as fh:
            fh.write(f"{time.strftime('%H:%M:%S')} {msg}\n")
    except OSError:
        pass


def to_dev(a: np.ndarray):
    import torch
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def idx_np(t) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def val_np(t) -> np.ndarray:
    return t.cpu().numpy()


def bits_equal(a: np.ndarray, b: np.ndarray) -> bool:
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    return a.shape == b.shape and np.array_equal(a.view(np.uint32), b.view(np.uint32))


def first_diff(a: np.ndarray, b: np.ndarray) -> str:
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    if a.shape != b.shape:
        return f"shape {a.shape} vs {b.shape}"
    av = a.view(np.uint32) if a.dtype == np.float32 else a
    bv = b.view(np.uint32) if b.dtype == np.float32 else b
    bad = np.argwhere(av != bv)
    if bad.size == 0:
        return "equal"
    p = tuple(bad[0])
    return f"{len(bad)} diffs, first at {p}: {a[p]!r} vs {b[p]!r}"


class Device:
    """Device buffers of one (P, m, k) problem and the calls on them."""

    def __init__(self, P: int, m: int, k: int, stride=None):
        import torch
        from paper_1901_04359_amd import binding as B
        self.B, self.torch = B, torch
        self.P, self.m, self.k = P, m, k
        self.stride = m if stride is None else stride
        self.grad_buf = torch.zeros(P * self.stride + 8, dtype=torch.float32, device="cuda")
        self.res_buf = torch.zeros(P * self.stride + 8, dtype=torch.float32, device="cuda")
        self.grad = self.grad_buf[: P * self.stride].view(P, self.stride)[:, :m]
        self.res = self.res_buf[: P * self.stride].view(P, self.stride)[:, :m]
        self.loc_idx = torch.zeros((P, k), dtype=torch.int32, device="cuda")
        self.loc_val = torch.zeros((P, k), dtype=torch.float32, device="cuda")
        self.g_idx = torch.zeros(k, dtype=torch.int32, device="cuda")
        self.g_val = torch.zeros(k, dtype=torch.float32, device="cuda")
        self.ws = B.alloc_workspace(m, k, P)
        # a dirty workspace must not matter
        self.ws.fill_(0xA5)
        # thresholds carried from call to call (gtopk_step_carry): zero = start from a sample
        self.thr_state = torch.zeros((P, 4), dtype=torch.int32, device="cuda")

    def set_grad(self, g: np.ndarray):
        self.grad.copy_(self.torch.from_numpy(np.ascontiguousarray(g)))

    def set_res(self, r: np.ndarray):
        self.res.copy_(self.torch.from_numpy(np.ascontiguousarray(r)))

    def residual(self) -> np.ndarray:
        return self.res.cpu().numpy()

    def local_select(self):
        self.B.gtopk_local_select(self.grad, self.res, self.k, self.loc_idx, self.loc_val, self.ws)
        self.torch.cuda.synchronize()
        return idx_np(self.loc_idx), val_np(self.loc_val)

    def tree(self):
        self.B.gtopk_tree(self.loc_idx, self.loc_val, self.P, self.k, self.g_idx, self.g_val, self.ws)
        self.torch.cuda.synchronize()
        return idx_np(self.g_idx), val_np(self.g_val)

    def restore(self):
        self.B.gtopk_residual_restore(self.res, self.k, self.loc_idx, self.loc_val, self.g_idx)
        self.torch.cuda.synchronize()

    def step_carry(self, want_loc=True):
        self.B.gtopk_step_carry(self.grad, self.res, self.k, self.g_idx, self.g_val,
                                self.loc_idx if want_loc else None,
                                self.loc_val if want_loc else None, self.thr_state, self.ws)
        self.torch.cuda.synchronize()
        return idx_np(self.g_idx), val_np(self.g_val)

    def carry_modes(self):
        """Per worker: 0 nothing known, 1 learning (next call samples), 2 next call skips sampling."""
        return self.thr_state[:, 0].cpu().numpy().tolist()

    def step(self, want_loc=True):
        self.B.gtopk_step(self.grad, self.res, self.k, self.g_idx, self.g_val,
                          self.loc_idx if want_loc else None, self.loc_val if want_loc else None,
                          self.ws)
        self.torch.cuda.synchronize()
        return idx_np(self.g_idx), val_np(self.g_val)
