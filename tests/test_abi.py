"""Host-side checks of the C-ABI library: it loads, exports every function the
header declares, sizes its workspace, and turns bad arguments into error codes
without touching a GPU.  No compute call is made here."""
import ctypes
import os
import re

import pytest

from paper_1901_04359_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "gtopk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gtopk_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    names = header_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings():
    for code in (0, -1, -2, -3, -4, -99):
        assert B.status_string(code).startswith("GTOPK")


def test_workspace_query():
    assert B.gtopk_workspace_bytes(65536, 66, 4) > 0
    big = B.gtopk_workspace_bytes(25_557_032, 255_570, 32)
    small = B.gtopk_workspace_bytes(25_557_032, 25_557, 32)
    assert big > small > 0
    assert big < 2 * 1024**3
    # invalid sizes give 0
    assert B.gtopk_workspace_bytes(0, 1, 1) == 0
    assert B.gtopk_workspace_bytes(100, 0, 1) == 0
    assert B.gtopk_workspace_bytes(100, 101, 1) == 0
    assert B.gtopk_workspace_bytes(100, 10, 3) == 0          # P not a power of two
    assert B.gtopk_workspace_bytes(2**31 + 1, 10, 2) == 0
    assert B.gtopk_merge_workspace_bytes(10, 0) == 0
    assert B.gtopk_merge_workspace_bytes(0, 1) == 0
    assert B.gtopk_merge_workspace_bytes(10, 3) > 0


FAKE = ctypes.c_void_p(0x10000)        # aligned, never dereferenced: every call below is rejected
ODD = ctypes.c_void_p(0x10004)


def test_argument_errors_local_select_and_step():
    lib = B.load()
    ok_ws = B.gtopk_workspace_bytes(1000, 10, 2)
    sel = lambda **kw: lib.gtopk_local_select(
        kw.get("grad", FAKE), kw.get("res", FAKE), kw.get("m", 1000), kw.get("stride", 1000),
        kw.get("P", 2), kw.get("k", 10), FAKE, FAKE, kw.get("ws", FAKE), kw.get("wsb", ok_ws), None)
    assert sel(grad=None) == B.GTOPK_EINVAL
    assert sel(ws=None) == B.GTOPK_EINVAL
    assert sel(m=0) == B.GTOPK_EINVAL
    assert sel(k=0) == B.GTOPK_EINVAL
    assert sel(k=1001) == B.GTOPK_EINVAL
    assert sel(P=3) == B.GTOPK_EINVAL
    assert sel(P=0) == B.GTOPK_EINVAL
    assert sel(stride=999) == B.GTOPK_EINVAL
    assert sel(res=ODD) == B.GTOPK_EALIGN
    assert sel(wsb=ok_ws - 1) == B.GTOPK_EWORKSPACE
    step = lambda **kw: lib.gtopk_step(
        FAKE, FAKE, 1000, 1000, kw.get("P", 2), 10, FAKE, FAKE, kw.get("li", FAKE),
        kw.get("lv", FAKE), FAKE, kw.get("wsb", ok_ws), None)
    assert step(P=6) == B.GTOPK_EINVAL
    assert step(li=None) == B.GTOPK_EINVAL          # loc_idx and loc_val go together
    assert step(wsb=0) == B.GTOPK_EWORKSPACE
    assert step(li=ODD) == B.GTOPK_EALIGN


def test_argument_errors_merge_tree_restore():
    lib = B.load()
    mws = B.gtopk_merge_workspace_bytes(10, 2)
    mg = lambda **kw: lib.gtopk_merge(
        kw.get("a", FAKE), FAKE, FAKE, FAKE, kw.get("k", 10), kw.get("batch", 2),
        kw.get("ins", 10), FAKE, FAKE, kw.get("outs", 10), FAKE, kw.get("wsb", mws), None)
    assert mg(a=None) == B.GTOPK_EINVAL
    assert mg(k=0) == B.GTOPK_EINVAL
    assert mg(batch=0) == B.GTOPK_EINVAL
    assert mg(ins=9) == B.GTOPK_EINVAL
    assert mg(outs=9) == B.GTOPK_EINVAL
    assert mg(a=ODD) == B.GTOPK_EALIGN
    assert mg(wsb=mws - 1) == B.GTOPK_EWORKSPACE
    tws = B.gtopk_workspace_bytes(10, 10, 4)
    tr = lambda **kw: lib.gtopk_tree(FAKE, FAKE, kw.get("P", 4), kw.get("k", 10), FAKE,
                                     kw.get("gv", FAKE), FAKE, kw.get("wsb", tws), None)
    assert tr(P=5) == B.GTOPK_EINVAL
    assert tr(k=0) == B.GTOPK_EINVAL
    assert tr(gv=None) == B.GTOPK_EINVAL
    assert tr(wsb=16) == B.GTOPK_EWORKSPACE
    rs = lambda **kw: lib.gtopk_residual_restore(
        kw.get("res", FAKE), kw.get("m", 100), kw.get("stride", 100), kw.get("P", 2),
        kw.get("k", 10), FAKE, FAKE, kw.get("g", FAKE), None)
    assert rs(res=None) == B.GTOPK_EINVAL
    assert rs(stride=99) == B.GTOPK_EINVAL
    assert rs(k=101) == B.GTOPK_EINVAL
    assert rs(g=ODD) == B.GTOPK_EALIGN


def test_binding_refuses_cpu_tensors():
    import torch
    t = torch.zeros(2, 8)
    with pytest.raises(TypeError):
        B.gtopk_residual_restore(t, 1, t.int(), t, t.int())


def test_argument_errors_apply_and_mask():
    lib = B.load()
    ap = lambda **kw: lib.gtopk_apply_update(
        kw.get("w", FAKE), kw.get("m", 100), kw.get("stride", 100), kw.get("copies", 1),
        kw.get("k", 10), FAKE, kw.get("gv", FAKE), ctypes.c_float(0.1), None)
    assert ap(w=None) == B.GTOPK_EINVAL
    assert ap(k=101) == B.GTOPK_EINVAL
    assert ap(copies=0) == B.GTOPK_EINVAL
    assert ap(stride=10) == B.GTOPK_EINVAL
    assert ap(gv=ODD) == B.GTOPK_EALIGN
    mk = lambda **kw: lib.gtopk_dense_mask(kw.get("g", FAKE), kw.get("k", 10), kw.get("m", 100),
                                           kw.get("mask", FAKE), None)
    assert mk(g=None) == B.GTOPK_EINVAL
    assert mk(k=0) == B.GTOPK_EINVAL
    assert mk(m=5) == B.GTOPK_EINVAL
    assert mk(mask=ODD) == B.GTOPK_EALIGN


def test_argument_errors_allreduce_and_dense_topk():
    lib = B.load()
    assert B.gtopk_allreduce_workspace_bytes(25_557_032, 32) >= 32 * (25_557_032 // 8192 + 2) * 4
    assert B.gtopk_allreduce_workspace_bytes(100, 3) > 0          # any P up to 1024
    assert B.gtopk_allreduce_workspace_bytes(100, 1025) == 0
    assert B.gtopk_allreduce_workspace_bytes(0, 2) == 0
    ok_ws = B.gtopk_allreduce_workspace_bytes(1000, 3)
    ar = lambda **kw: lib.gtopk_topk_allreduce(
        kw.get("li", FAKE), FAKE, kw.get("P", 3), kw.get("k", 10), kw.get("m", 1000),
        kw.get("dense", FAKE), kw.get("ws", FAKE), kw.get("wsb", ok_ws), None)
    assert ar(li=None) == B.GTOPK_EINVAL
    assert ar(P=0) == B.GTOPK_EINVAL
    assert ar(P=1025) == B.GTOPK_EINVAL
    assert ar(k=1001) == B.GTOPK_EINVAL
    assert ar(dense=ODD) == B.GTOPK_EALIGN
    assert ar(wsb=ok_ws - 1) == B.GTOPK_EWORKSPACE
    ok_ws = B.gtopk_workspace_bytes(1000, 10, 1)
    dt = lambda **kw: lib.gtopk_dense_topk(
        kw.get("dense", FAKE), kw.get("m", 1000), kw.get("k", 10), kw.get("gi", FAKE), FAKE,
        kw.get("ws", FAKE), kw.get("wsb", ok_ws), None)
    assert dt(dense=None) == B.GTOPK_EINVAL
    assert dt(k=0) == B.GTOPK_EINVAL
    assert dt(k=1001) == B.GTOPK_EINVAL
    assert dt(gi=ODD) == B.GTOPK_EALIGN
    assert dt(wsb=ok_ws - 1) == B.GTOPK_EWORKSPACE
    # merged pairs have 2k slots in a uint32
    assert B.gtopk_merge_workspace_bytes(2**30 + 1, 1) == 0
    assert B.gtopk_workspace_bytes(2**31, 2**30 + 1, 2) == 0
