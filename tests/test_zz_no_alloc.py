"""gtopk_step_static (the entry point for callers that cannot allocate: its workspace is a
device array inside the library) against gtopk_step with a caller-owned workspace, through
the C ABI, bit for bit, on two calls in a row, the second with a smaller input, and both
against the oracle.  Runs last in the suite and must also pass alone in a fresh process."""
import numpy as np
import pytest

from oracle import gtopk_oracle as orc
from paper_1901_04359_amd import workloads as W
from tests.gpu_harness import Device, bits_equal, first_diff, say, idx_np, val_np

pytestmark = pytest.mark.gpu


def run_static(dev, want_loc=True):
    dev.B.gtopk_step_static(dev.grad, dev.res, dev.k, dev.g_idx, dev.g_val,
                            dev.loc_idx if want_loc else None, dev.loc_val if want_loc else None)
    dev.torch.cuda.synchronize()
    return idx_np(dev.g_idx), val_np(dev.g_val)


def test_static_workspace_matches_gtopk_step_twice_in_a_row():
    from paper_1901_04359_amd import binding as B
    # first call: the ResNet-20-sized configuration; second call: a smaller problem, so the
    # array still holds the first call's state beyond what the second one uses
    shapes = [("C2", W.CONFIGS["C2"]), ("C1", W.CONFIGS["C1"])]
    for name, cfg in shapes:
        P, m, k = cfg.P, cfg.m, cfg.k
        assert B.gtopk_workspace_bytes(m, k, P) <= B.STATIC_WORKSPACE_BYTES
        a = Device(P, m, k)          # caller-owned workspace (dirty on purpose, see Device)
        b = Device(P, m, k)          # its workspace tensor is not used by the static call
        res = np.zeros((P, m), dtype=np.float32)
        for it in range(2):
            g = W.gradients(cfg, it)
            for dev in (a, b):
                dev.set_res(res)
                dev.set_grad(g)
            say(f"no-alloc {name} it={it}: gtopk_step")
            gi_a, gv_a = a.step()
            say(f"no-alloc {name} it={it}: gtopk_step_static")
            gi_b, gv_b = run_static(b)
            assert np.array_equal(gi_a, gi_b), first_diff(gi_a, gi_b)
            assert bits_equal(gv_a, gv_b), first_diff(gv_a, gv_b)
            assert np.array_equal(idx_np(a.loc_idx), idx_np(b.loc_idx))
            assert bits_equal(val_np(a.loc_val), val_np(b.loc_val))
            ra, rb = a.residual(), b.residual()
            assert bits_equal(ra, rb), first_diff(ra, rb)
            exp = orc.step(res, g, k)
            assert np.array_equal(gi_b, exp["g_idx"]) and bits_equal(gv_b, exp["g_val"])
            assert bits_equal(rb, exp["residual"])
            res = exp["residual"]


def test_static_workspace_rejects_sizes_beyond_its_array():
    """A problem whose workspace does not fit the array is refused on the host, before
    anything is enqueued."""
    import torch
    from paper_1901_04359_amd import binding as B
    P, m, k = 16, 2_000_000, 20_000
    assert B.gtopk_workspace_bytes(m, k, P) > B.STATIC_WORKSPACE_BYTES
    grad = torch.zeros((P, m), dtype=torch.float32, device="cuda")
    res = torch.full((P, m), 3.0, dtype=torch.float32, device="cuda")
    g_idx = torch.full((k,), -1, dtype=torch.int32, device="cuda")
    g_val = torch.zeros(k, dtype=torch.float32, device="cuda")
    say("no-alloc: oversize call must be refused")
    with pytest.raises(B.GtopkError) as err:
        B.gtopk_step_static(grad, res, k, g_idx, g_val, None, None)
    assert err.value.status == B.GTOPK_EWORKSPACE
    torch.cuda.synchronize()
    assert bool((res == 3.0).all()) and bool((g_idx == -1).all())
