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


def test_argument_errors_timed_probe():
    lib = B.load()
    ws = B.gtopk_workspace_bytes(1000, 10, 2)
    assert lib.gtopk_step_timed(FAKE, FAKE, 1000, 1000, 2, 10, FAKE, FAKE, FAKE, FAKE, None, FAKE,
                                ws, None, None) == B.GTOPK_EINVAL
    ev = (ctypes.c_void_p * 6)(1, 2, 3, 0, 5, 6)               # one NULL handle
    assert lib.gtopk_step_timed(FAKE, FAKE, 1000, 1000, 2, 10, FAKE, FAKE, FAKE, FAKE, None, FAKE,
                                ws, None, ev) == B.GTOPK_EINVAL
    carry = lambda **kw: lib.gtopk_step_carry(FAKE, FAKE, 1000, 1000, kw.get("P", 2), 10, FAKE, FAKE,
                                              FAKE, FAKE, kw.get("state", FAKE), FAKE,
                                              kw.get("wsb", ws), None)
    assert carry(state=None) == B.GTOPK_EINVAL
    assert carry(state=ODD) == B.GTOPK_EALIGN
    assert carry(P=3) == B.GTOPK_EINVAL
    assert carry(wsb=8) == B.GTOPK_EWORKSPACE
    pr = lambda **kw: lib.gtopk_probe_stream(kw.get("a", FAKE), FAKE, kw.get("n", 32768),
                                             kw.get("mode", 0), kw.get("sink", FAKE), None)
    assert pr(a=None) == B.GTOPK_EINVAL
    assert pr(n=1000) == B.GTOPK_EINVAL                         # not a multiple of 32768
    assert pr(mode=8) == B.GTOPK_EINVAL and pr(mode=-1) == B.GTOPK_EINVAL
    assert pr(mode=1, sink=None) == B.GTOPK_EINVAL
    assert pr(a=ODD) == B.GTOPK_EALIGN


def test_debug_plan_describes_the_sampler():
    plan = B.gtopk_debug_plan(25_557_032, 25_557, 32)
    assert plan["tile_len"] == 64 and plan["n_tiles"] >= 4096
    assert (plan["n_tiles"] - 1) * plan["tile_stride"] < 25_557_032 <= plan["n_tiles"] * plan["tile_stride"]
    assert plan["tile_stride"] >= plan["tile_len"]
    assert 256 <= plan["target"] < plan["n_tiles"] * plan["tile_len"]
    assert 25_557 < plan["capacity"] <= 25_557_032
    # a short row is sampled whole: the "sample" is an exact count
    small = B.gtopk_debug_plan(5000, 50, 2)
    assert small["tile_stride"] == small["tile_len"] and small["target"] == 50
    with pytest.raises(B.GtopkError):
        B.gtopk_debug_plan(100, 0, 2)
    # which sizes gtopk_step runs as its few-launch path for small problems
    c1 = B.gtopk_debug_plan(65_536, 66, 4)
    assert c1["small_path"] == 1
    # the few-launch path samples less: one block per worker reads it
    assert 0 < c1["small_n_tiles"] * c1["tile_len"] <= c1["n_tiles"] * c1["tile_len"]
    assert c1["small_target"] >= 1 and c1["small_tile_stride"] >= c1["tile_len"]
    assert B.gtopk_debug_plan(14_728_266, 14_728, 16)["small_n_tiles"] == 0
    # merges of very large sets go through a speculative threshold
    assert B.gtopk_debug_plan(25_557_032, 255_570, 32)["merge_filtered"] == 0
    big = B.gtopk_debug_plan(25_557_032, 6_389_258, 32)
    assert big["merge_filtered"] == 1 and big["merge_n_tiles"] * big["tile_len"] < 6_389_258
    assert B.gtopk_debug_plan(25_557_032, 6_389_258, 1)["merge_filtered"] == 0      # P = 1: no merge
    # long runs of candidates (C4b and the warm-up densities) are selected in place
    assert B.gtopk_debug_plan(25_557_032, 25_557, 32)["run_groups"] == 0
    assert B.gtopk_debug_plan(25_557_032, 255_570, 32)["run_groups"] == 1
    assert B.gtopk_debug_plan(25_557_032, 6_389_258, 32)["run_groups"] == 1
    assert B.gtopk_debug_plan(269_722, 270, 8)["small_path"] == 1
    assert B.gtopk_debug_plan(14_728_266, 14_728, 16)["small_path"] == 0
    assert B.gtopk_debug_plan(100_000, 513, 2)["small_path"] == 0
    assert B.gtopk_debug_plan(100_000, 100, 128)["small_path"] == 0
    assert B.gtopk_debug_plan(1_048_574, 10, 2)["small_path"] == 0


def test_argument_errors_step_static():
    lib = B.load()
    st = lambda **kw: lib.gtopk_step_static(
        kw.get("grad", FAKE), FAKE, kw.get("m", 1000), kw.get("stride", 1000), kw.get("P", 2),
        kw.get("k", 10), FAKE, FAKE, FAKE, FAKE, None)
    assert st(P=3) == B.GTOPK_EINVAL
    assert st(k=0) == B.GTOPK_EINVAL
    # a problem whose workspace exceeds the library's static array is refused on the host
    assert B.gtopk_workspace_bytes(25_557_032, 25_557, 32) > B.STATIC_WORKSPACE_BYTES
    assert st(m=25_557_032, stride=25_557_032, P=32, k=25_557) == B.GTOPK_EWORKSPACE
    assert B.gtopk_workspace_bytes(269_722, 270, 8) <= B.STATIC_WORKSPACE_BYTES
