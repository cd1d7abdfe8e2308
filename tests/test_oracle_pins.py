"""Pins for the CPU oracle: every check here is written against what the paper
and the mathematics fix, in code that shares nothing with oracle/ (pure-Python
brute force, dense definitions, library top-k, closed forms, a hand-worked
example), and the last test plants mistakes in the oracle to show that the
pins notice them.  The paper prints no numeric worked example (its example
figures are images), so no value below is quoted from it."""
import json
import math
import os
import struct

import numpy as np
import pytest

from oracle import gtopk_oracle as orc
from paper_1901_04359_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
f32 = np.float32


# --------------------------------------------------------------------------
# independent brute-force definitions (pure Python, no oracle code)
# --------------------------------------------------------------------------

def brute_first_k(values, indices, k):
    """Repeated arg-max under (|v| descending, index ascending).  `values` are
    Python floats (exact images of the float32 values), so abs() and > are exact."""
    left = list(zip(indices, values))
    chosen = []
    for _ in range(k):
        best = None
        for (i, v) in left:
            if best is None or abs(v) > abs(best[1]) or (abs(v) == abs(best[1]) and i < best[0]):
                best = (i, v)
        chosen.append(best)
        left.remove(best)
    chosen.sort(key=lambda t: t[0])
    return [c[0] for c in chosen], [c[1] for c in chosen]


def brute_local_select(res, grad, k):
    acc = [float(f32(f32(r) + f32(g))) for r, g in zip(res, grad)]
    idx, val = brute_first_k(acc, list(range(len(acc))), k)
    new = list(acc)
    for i in idx:
        new[i] = 0.0
    return idx, val, new, acc


def brute_merge_dense(m, a_idx, a_val, b_idx, b_val, k):
    """Definition 1 evaluated on dense length-m vectors with presence marks."""
    dense_a = [None] * m
    dense_b = [None] * m
    for i, v in zip(a_idx, a_val):
        dense_a[int(i)] = float(v)
    for i, v in zip(b_idx, b_val):
        dense_b[int(i)] = float(v)
    cand_i, cand_v = [], []
    for i in range(m):
        if dense_a[i] is not None and dense_b[i] is not None:
            cand_i.append(i)
            cand_v.append(float(f32(f32(dense_a[i]) + f32(dense_b[i]))))
        elif dense_a[i] is not None:
            cand_i.append(i)
            cand_v.append(dense_a[i])
        elif dense_b[i] is not None:
            cand_i.append(i)
            cand_v.append(dense_b[i])
    return brute_first_k(cand_v, cand_i, k)


def bits(x):
    return np.asarray(x, dtype=np.float32).view(np.uint32)


def same_bits(a, b):
    a = np.asarray(a, dtype=np.float32)
    b = np.asarray(b, dtype=np.float32)
    return a.shape == b.shape and np.array_equal(a.view(np.uint32), b.view(np.uint32))


def random_small(rng, m, kind):
    if kind == "gauss":
        return rng.standard_normal(m).astype(np.float32)
    if kind == "ties":      # few distinct magnitudes, both signs, some zeros
        return (rng.integers(-3, 4, m)).astype(np.float32) * f32(0.5)
    if kind == "special":
        return W.special_values(m, seed=int(rng.integers(0, 1000)))
    raise ValueError(kind)


# --------------------------------------------------------------------------
# the pins, as plain functions (the mutation test calls them again)
# --------------------------------------------------------------------------

def pin_local_select_bruteforce():
    rng = np.random.default_rng(11)
    for kind in ("gauss", "ties", "special"):
        for m, k in ((1, 1), (7, 1), (7, 7), (33, 5), (64, 17), (97, 40)):
            res = random_small(rng, m, kind)
            grad = random_small(rng, m, kind)
            idx, val, new = orc.local_select(res, grad, k)
            bi, bv, bnew, _ = brute_local_select(res.tolist(), grad.tolist(), k)
            assert idx.dtype == np.uint32 and idx.tolist() == bi, (kind, m, k)
            assert same_bits(val, np.array(bv, dtype=np.float32)), (kind, m, k)
            assert same_bits(new, np.array(bnew, dtype=np.float32)), (kind, m, k)


def pin_local_select_library_topk():
    """Tie-free input: the selected SET is unique, so a library top-k on |acc|
    must return the same set (numpy argpartition and torch.topk, both on CPU)."""
    import torch
    rng = np.random.default_rng(5)
    m, k = 20000, 157
    mags = rng.permutation(m).astype(np.float32) + f32(1.0)      # all distinct
    acc = mags * np.where(rng.random(m) < 0.5, -1, 1).astype(np.float32)
    res = (acc * f32(0.25)).astype(np.float32)
    grad = (acc * f32(0.75)).astype(np.float32)                  # 0.25x + 0.75x == x exactly
    assert np.array_equal(res + grad, acc)
    idx, val, _ = orc.local_select(res, grad, k)
    part = np.sort(np.argpartition(-np.abs(acc), k - 1)[:k])
    assert np.array_equal(idx, part)
    tk = torch.topk(torch.from_numpy(np.abs(acc)), k).indices.numpy()
    assert np.array_equal(idx, np.sort(tk))
    assert same_bits(val, acc[part])


def pin_local_select_invariants():
    cfg = W.scaled(W.CONFIGS["C2"], 50021, P=2)
    res = np.zeros((2, cfg.m), dtype=np.float32)
    for it in range(3):
        g = W.gradients(cfg, it, threads=1)
        for w in range(2):
            idx, val, new = orc.local_select(res[w], g[w], cfg.k)
            assert idx.shape == (cfg.k,) and val.shape == (cfg.k,)
            assert (np.diff(idx.astype(np.int64)) > 0).all()
            # conservation, exact: what was sent plus what was kept is g + r
            sent = np.zeros(cfg.m, dtype=np.float32)
            sent[idx] = val
            assert np.array_equal(sent + new, g[w] + res[w])
            # threshold property with the index rule at equality
            acc = g[w] + res[w]
            mag = np.abs(acc.astype(np.float64))
            selected = np.zeros(cfg.m, dtype=bool)
            selected[idx] = True
            lo = mag[selected].min()
            hi = mag[~selected].max()
            assert lo >= hi
            if lo == hi:
                assert idx[mag[idx] == lo].max() < np.nonzero((~selected) & (mag == hi))[0].min()
            res[w] = new


def pin_local_select_special_k():
    rng = np.random.default_rng(3)
    m = 50
    res = rng.standard_normal(m).astype(np.float32)
    grad = rng.standard_normal(m).astype(np.float32)
    acc = res + grad
    idx, val, new = orc.local_select(res, grad, m)          # k = m: everything goes
    assert idx.tolist() == list(range(m)) and same_bits(val, acc)
    assert same_bits(new, np.zeros(m, dtype=np.float32))    # all +0.0
    idx, val, new = orc.local_select(res, grad, 1)          # k = 1: the arg-max
    j = int(np.argmax(np.abs(acc)))
    assert idx.tolist() == [j] and same_bits(val, acc[j:j + 1])
    # zeroing writes +0.0 even over a negative value; -0.0 and +0.0 tie by index
    r0 = np.zeros(4, dtype=np.float32)
    g0 = np.array([-0.0, 0.0, -0.0, 0.0], dtype=np.float32)
    idx, val, new = orc.local_select(r0, g0, 2)
    assert idx.tolist() == [0, 1]
    # +0.0 + -0.0 = +0.0 in round-to-nearest, so every accumulated value is +0.0
    assert bits(val).tolist() == [0, 0]
    assert bits(new).tolist() == [0, 0, 0, 0]


def pin_denormals_not_flushed():
    tiny = np.array([struct.unpack("f", struct.pack("I", 0x00000003))[0]], dtype=np.float32)
    idx, val, _ = orc.local_select(tiny.copy(), tiny.copy(), 1)
    assert bits(val).tolist() == [0x00000006]
    # a denormal outranks zero, and a larger denormal outranks a smaller one
    g = np.zeros(5, dtype=np.float32)
    g.view(np.uint32)[1] = 0x00000001
    g.view(np.uint32)[3] = 0x80000002
    idx, val, _ = orc.local_select(np.zeros(5, dtype=np.float32), g, 2)
    assert idx.tolist() == [1, 3]
    idx, _, _ = orc.local_select(np.zeros(5, dtype=np.float32), g, 1)
    assert idx.tolist() == [3]


def pin_merge_dense_definition():
    rng = np.random.default_rng(17)
    for kind in ("gauss", "ties", "cancel"):
        for m, k in ((6, 3), (40, 7), (200, 50), (64, 32), (64, 64)):
            idx, val = W.ksets(2, k, m, seed=int(rng.integers(0, 10**6)), overlap=0.4,
                               value_kind=kind)
            oi, ov = orc.merge(idx[0], val[0], idx[1], val[1], k)
            bi, bv = brute_merge_dense(m, idx[0], val[0], idx[1], val[1], k)
            assert oi.dtype == np.uint32 and oi.tolist() == bi, (kind, m, k)
            assert same_bits(ov, np.array(bv, dtype=np.float32)), (kind, m, k)
            assert len(oi) == k and set(oi.tolist()) <= set(idx[0].tolist()) | set(idx[1].tolist())
            # commutative: operand order is irrelevant
            ci, cv = orc.merge(idx[1], val[1], idx[0], val[0], k)
            assert np.array_equal(ci, oi) and same_bits(cv, ov)


def pin_merge_special_supports():
    rng = np.random.default_rng(23)
    k = 25
    # identical supports: nothing can be dropped, output = elementwise fp32 sum
    ia = np.sort(rng.choice(1000, k, replace=False)).astype(np.uint32)
    va = rng.standard_normal(k).astype(np.float32)
    vb = rng.standard_normal(k).astype(np.float32)
    oi, ov = orc.merge(ia, va, ia.copy(), vb, k)
    assert np.array_equal(oi, ia) and same_bits(ov, va + vb)
    # disjoint supports: output = top-k of the concatenation, values untouched
    ib = (ia + np.uint32(1000)).astype(np.uint32)
    oi, ov = orc.merge(ia, va, ib, vb, k)
    cat_i = np.concatenate([ia, ib])
    cat_v = np.concatenate([va, vb])
    bi, bv = brute_first_k(cat_v.tolist(), cat_i.tolist(), k)
    assert oi.tolist() == bi and same_bits(ov, np.array(bv, dtype=np.float32))
    # R9: a single-owner -0.0 stays -0.0 (k = union size, so it must be kept)
    oi, ov = orc.merge(np.array([1, 5], dtype=np.uint32), np.array([-0.0, 2.0], dtype=np.float32),
                       np.array([5, 9], dtype=np.uint32), np.array([1.0, -0.0], dtype=np.float32), 2)
    assert oi.tolist() == [1, 5] and bits(ov).tolist() == [0x80000000, bits(f32(3.0)).tolist()]
    # R4: a sum that cancels to zero is still a candidate and ranks last
    oi, ov = orc.merge(np.array([2, 4], dtype=np.uint32), np.array([1.0, -8.0], dtype=np.float32),
                       np.array([4, 6], dtype=np.uint32), np.array([8.0, 0.5], dtype=np.float32), 2)
    assert oi.tolist() == [2, 6] and ov.tolist() == [1.0, 0.5]
    oi, ov = orc.merge(np.array([2, 4], dtype=np.uint32), np.array([1.0, -8.0], dtype=np.float32),
                       np.array([2, 4], dtype=np.uint32), np.array([-1.0, 8.0], dtype=np.float32), 2)
    assert oi.tolist() == [2, 4] and bits(ov).tolist() == [0, 0]


def pin_tree_p1_p2():
    rng = np.random.default_rng(29)
    m, k = 300, 40
    idx, val = W.ksets(2, k, m, seed=4, overlap=0.5)
    # P = 1: zero rounds, the result is the set itself divided by 1
    gi, gv = orc.tree([idx[0]], [val[0]], k)
    assert np.array_equal(gi, idx[0]) and same_bits(gv, val[0])
    # P = 2: top-k of the dense sum of the two sparse vectors, halved
    gi, gv = orc.tree([idx[0], idx[1]], [val[0], val[1]], k)
    bi, bv = brute_merge_dense(m, idx[0], val[0], idx[1], val[1], k)
    assert gi.tolist() == bi
    assert same_bits(gv, np.array(bv, dtype=np.float32) * f32(0.5))


def pin_tree_shared_support():
    """All P workers hold one index set: no merge can drop anything, so the
    result is the pairwise-tree fp32 sum at those indices, divided by P."""
    rng = np.random.default_rng(31)
    for P in (4, 8):
        k = 19
        ia = np.sort(rng.choice(500, k, replace=False)).astype(np.uint32)
        vals = [rng.standard_normal(k).astype(np.float32) for _ in range(P)]
        gi, gv = orc.tree([ia] * P, vals, k)
        level = list(vals)
        while len(level) > 1:
            level = [(level[2 * i] + level[2 * i + 1]).astype(np.float32)
                     for i in range(len(level) // 2)]
        assert np.array_equal(gi, ia)
        assert same_bits(gv, level[0] / f32(P))


def pin_tree_order_by_composition():
    """P = 4 and P = 8 written out by hand as nested merges in the tree order:
    round 0 merges (0,1) (2,3) (4,5) (6,7), round 1 merges (0,2) (4,6), round 2 (0,4)."""
    m, k = 400, 30
    idx, val = W.ksets(8, k, m, seed=9, overlap=0.5, value_kind="cancel")
    mg = lambda a, b: brute_merge_dense(m, a[0], a[1], b[0], b[1], k)
    s = [(idx[w].tolist(), val[w].tolist()) for w in range(8)]
    r01, r23, r45, r67 = mg(s[0], s[1]), mg(s[2], s[3]), mg(s[4], s[5]), mg(s[6], s[7])
    r0123, r4567 = mg(r01, r23), mg(r45, r67)
    top = mg(r0123, r4567)
    gi, gv = orc.tree(list(idx[:4]), list(val[:4]), k)
    assert gi.tolist() == r0123[0]
    assert same_bits(gv, np.array(r0123[1], dtype=np.float32) / f32(4))
    gi, gv = orc.tree(list(idx), list(val), k)
    assert gi.tolist() == top[0]
    assert same_bits(gv, np.array(top[1], dtype=np.float32) / f32(8))
    # structure: log2 P rounds, P - 1 merges, rank 0 active in every round
    hist = orc.tree_rounds(list(idx), list(val), k)
    assert len(hist) == 3
    active = [sum(1 for c in rnd if c is not None) for rnd in hist]
    assert active == [4, 2, 1]
    assert all(rnd[0] is not None for rnd in hist)
    assert sum(8 >> (j + 1) for j in range(3)) == 7


def pin_tree_not_the_dense_topk():
    """The tree is a heuristic: for P > 2 it may differ from the top-k of the
    P-way dense sum, because a value dropped in an early round never reaches a
    later sum.  Three values of 2 at one index lose to single 3s round by round."""
    k = 1
    idx = [np.array([i], dtype=np.uint32) for i in (0, 1, 0, 2)]
    val = [np.array([v], dtype=np.float32) for v in (2.0, 3.0, 2.0, 3.5)]
    gi, gv = orc.tree(idx, val, k)
    assert gi.tolist() == [2] and gv.tolist() == [3.5 / 4]       # dense sum would pick index 0 (4.0)


def pin_average_is_exact_scale():
    idx, val = W.ksets(4, 16, 100, seed=2, overlap=1.0)           # all share the support
    undiv = orc.tree_rounds(list(idx), list(val), 16)[-1][0][1]
    _, gv = orc.tree(list(idx), list(val), 16)
    assert same_bits(gv * f32(4), undiv)
    assert same_bits(gv, undiv * f32(0.25))


def pin_restore_closed_form():
    rng = np.random.default_rng(37)
    m, k = 500, 60
    res = rng.standard_normal(m).astype(np.float32)
    grad = rng.standard_normal(m).astype(np.float32)
    acc = res + grad
    idx, val, after = orc.local_select(res, grad, k)
    g_idx = np.sort(np.concatenate([idx[::3], np.setdiff1d(np.arange(m), idx)[:k - len(idx[::3])]])
                    ).astype(np.uint32)
    out = orc.residual_restore(after, idx, val, g_idx)
    expect = acc.copy()
    for i in idx.tolist():
        if i in set(g_idx.tolist()):
            expect[i] = 0.0
    assert same_bits(out, expect)
    # nothing outside the local set moves
    untouched = np.ones(m, dtype=bool)
    untouched[idx] = False
    assert same_bits(out[untouched], after[untouched])
    # R8: a locally selected -0.0 that is restored becomes +0.0 (literal add onto +0.0)
    r = orc.residual_restore(np.zeros(3, dtype=np.float32), np.array([1], dtype=np.uint32),
                             np.array([-0.0], dtype=np.float32), np.array([2], dtype=np.uint32))
    assert bits(r).tolist() == [0, 0, 0]


def pin_hand_worked_example():
    with open(os.path.join(GOLDEN, "hand_worked_p4_k2.json")) as fh:
        ex = json.load(fh)
    P, m, k = ex["P"], ex["m"], ex["k"]
    grad = np.array(ex["grad"], dtype=np.float32)
    res = np.zeros((P, m), dtype=np.float32)
    out = orc.step(res, grad, k)
    assert out["loc_idx"].tolist() == ex["loc_idx"]
    assert out["loc_val"].tolist() == ex["loc_val"]
    assert np.array_equal(out["residual_after_select"], np.array(ex["residual_after_select"], dtype=np.float32))
    hist = orc.tree_rounds(list(out["loc_idx"]), list(out["loc_val"]), k)
    for rnd, name in ((hist[0], "round0"), (hist[1], "round1")):
        for rank, want in ex[name].items():
            got = rnd[int(rank)]
            assert got[0].tolist() == want["idx"] and got[1].tolist() == want["val"]
        assert sum(1 for c in rnd if c is not None) == len(ex[name])
    assert out["g_idx"].tolist() == ex["g_idx"]
    assert out["g_val"].tolist() == ex["g_val"]
    assert np.array_equal(out["residual"], np.array(ex["residual"], dtype=np.float32))
    # the same local sets through Algorithm 1's all-reduce and Algorithm 2's second top-k
    dense = orc.topk_allreduce(list(out["loc_idx"]), list(out["loc_val"]), m)
    assert dense.tolist() == ex["alg1_dense"]
    n_idx, n_val = orc.dense_topk(dense, k)
    assert n_idx.tolist() == ex["alg2_g_idx"] and n_val.tolist() == ex["alg2_g_val"]
    for w in range(P):
        r = orc.residual_restore(out["residual_after_select"][w], out["loc_idx"][w],
                                 out["loc_val"][w], n_idx)
        assert r.tolist() == ex["alg2_residual"][w]


def pin_step_feedback_and_bounds():
    """Multi-iteration: per-worker conservation through the residual feedback,
    global set inside the union of the local sets, union size within [k, kP]."""
    cfg = W.CONFIGS["C1"]
    P, m, k = cfg.P, cfg.m, cfg.k
    res = np.zeros((P, m), dtype=np.float32)
    for it in range(cfg.iters):
        g = W.gradients(cfg, it, threads=1)
        out = orc.step(res, g, k)
        acc = res + g
        union = set()
        gset = set(out["g_idx"].tolist())
        for w in range(P):
            loc = out["loc_idx"][w]
            union |= set(loc.tolist())
            expect = acc[w].copy()
            both = [i for i in loc.tolist() if i in gset]
            expect[both] = 0.0
            assert same_bits(out["residual"][w], expect)
        assert gset <= union and k <= len(union) <= k * P
        assert len(out["g_idx"]) == k and (np.diff(out["g_idx"].astype(np.int64)) > 0).all()
        res = out["residual"]


def pin_apply_update_and_mask():
    """Model update against per-element Python arithmetic with explicit float32 rounding of
    each of the two operations; eta = 0 leaves W unchanged; a power-of-two eta is exact."""
    rng = np.random.default_rng(41)
    m, k = 300, 37
    Wt = rng.standard_normal(m).astype(np.float32)
    g_idx = np.sort(rng.choice(m, k, replace=False)).astype(np.uint32)
    g_val = rng.standard_normal(k).astype(np.float32)
    for lr in (0.1, 0.01, 1.0, 0.0, 0.25):
        out = orc.apply_update(Wt, g_idx, g_val, lr)
        exp = Wt.copy()
        for i, v in zip(g_idx.tolist(), g_val.tolist()):
            p = f32(f32(lr) * f32(v))
            exp[i] = f32(f32(exp[i]) - p)
        assert same_bits(out, exp), lr
        untouched = np.ones(m, dtype=bool)
        untouched[g_idx] = False
        assert same_bits(out[untouched], Wt[untouched])
    assert same_bits(orc.apply_update(Wt, g_idx, g_val, 0.0), Wt)
    quarter = orc.apply_update(np.zeros(m, dtype=np.float32), g_idx, g_val, 0.25)
    assert same_bits(quarter[g_idx] * f32(-4), g_val)
    mask = orc.dense_mask(g_idx, m)
    assert mask.dtype == np.uint8 and mask.sum() == k
    assert [i for i in range(m) if mask[i]] == g_idx.tolist()


def pin_topk_allreduce():
    """Algorithm 1's TopKAllReduce: per-index Python loop; integer-valued inputs (every fp32
    sum exact, so a float64 scatter-add must agree); an order-sensitive input; -0.0."""
    rng = np.random.default_rng(51)
    m, k, P = 97, 13, 4
    idx, val = [], []
    for g in range(P):
        idx.append(np.sort(rng.choice(m // 2, k, replace=False)).astype(np.uint32))   # many shared
        val.append((rng.standard_normal(k) * 10.0 ** rng.integers(-3, 4, k)).astype(np.float32))
    out = orc.topk_allreduce(idx, val, m)
    exp = np.zeros(m, dtype=np.float32)
    for i in range(m):
        acc = f32(0.0)
        for g in range(P):
            for t in range(k):
                if int(idx[g][t]) == i:
                    acc = f32(acc + val[g][t])
        exp[i] = f32(acc / f32(P))
    assert out.dtype == np.float32 and same_bits(out, exp)
    # integer-valued: exact in any precision
    ival = [rng.integers(-1000, 1000, k).astype(np.float32) for _ in range(P)]
    ref = np.zeros(m, dtype=np.float64)
    for g in range(P):
        np.add.at(ref, idx[g], ival[g].astype(np.float64))
    assert np.array_equal(orc.topk_allreduce(idx, ival, m).astype(np.float64), ref / P)
    # rank order of the adds: ((1 + 1e8) - 1e8) = 0 in fp32; adding the 1 last gives 1
    one = [np.array([5], dtype=np.uint32)] * 3 + [np.array([6], dtype=np.uint32)]
    v = [np.array([x], dtype=np.float32) for x in (1.0, 1e8, -1e8, 8.0)]
    r = orc.topk_allreduce(one, v, 8)
    assert r[5] == 0.0 and r[6] == 2.0 and not r[[0, 1, 2, 3, 4, 7]].any()
    # literal += on a zero vector: a lone -0.0 becomes +0.0
    z = orc.topk_allreduce([np.array([2], dtype=np.uint32)], [np.array([-0.0], dtype=np.float32)], 4)
    assert bits(z).tolist() == [0, 0, 0, 0]
    # P = 1: the scatter itself
    s1 = orc.topk_allreduce(idx[:1], val[:1], m)
    assert same_bits(s1[idx[0]], val[0]) and np.count_nonzero(s1) == np.count_nonzero(val[0])


def pin_dense_topk_and_p2_equals_tree():
    """Top-k of a dense vector: brute force, library top-k, fewer than k non-zeros; and for
    P = 2 the naive aggregation (Algorithm 2) must equal the tree (Algorithm 3)."""
    rng = np.random.default_rng(52)
    for kind in ("gauss", "ties", "special"):
        m, k = 60, 9
        d = random_small(rng, m, kind)
        oi, ov = orc.dense_topk(d, k)
        bi, _ = brute_first_k([float(x) for x in d], list(range(m)), k)
        assert oi.tolist() == bi and same_bits(ov, d[oi])
    import torch
    d = rng.standard_normal(5000).astype(np.float32)
    oi, _ = orc.dense_topk(d, 50)
    assert set(oi.tolist()) == set(torch.topk(torch.from_numpy(np.abs(d)), 50).indices.tolist())
    oi, ov = orc.dense_topk(np.array([0, 5, 0, 0, -3], dtype=np.float32), 4)
    assert oi.tolist() == [0, 1, 2, 4] and ov.tolist() == [0, 5, 0, -3]
    for seed in range(5):
        r2 = np.random.default_rng(seed)
        m, k = 200, 17
        idx = [np.sort(r2.choice(m, k, replace=False)).astype(np.uint32) for _ in range(2)]
        val = [r2.standard_normal(k).astype(np.float32) for _ in range(2)]
        ti, tv = orc.tree(idx, val, k)
        ni, nv = orc.dense_topk(orc.topk_allreduce(idx, val, m), k)
        # candidates of the dense top-k also include untouched zeros; with >= k non-zero
        # sums they never win
        assert ni.tolist() == ti.tolist() and same_bits(nv, tv)


def _mut_allreduce_reverse_order(loc_idx, loc_val, m):
    dense = np.zeros(m, dtype=np.float32)
    for g in reversed(range(len(loc_idx))):
        dense[loc_idx[g]] = (dense[loc_idx[g]] + loc_val[g]).astype(np.float32)
    return (dense / np.float32(len(loc_idx))).astype(np.float32)


def _mut_allreduce_no_average(loc_idx, loc_val, m):
    dense = np.zeros(m, dtype=np.float32)
    for g in range(len(loc_idx)):
        dense[loc_idx[g]] = (dense[loc_idx[g]] + loc_val[g]).astype(np.float32)
    return dense


def _mut_allreduce_own_twice(loc_idx, loc_val, m):
    dense = np.zeros(m, dtype=np.float32)
    dense[loc_idx[0]] = loc_val[0]                       # the printed initialisation, literally
    for g in range(len(loc_idx)):
        dense[loc_idx[g]] = (dense[loc_idx[g]] + loc_val[g]).astype(np.float32)
    return (dense / np.float32(len(loc_idx))).astype(np.float32)


def _mut_dense_topk_signed(dense, k):
    order = np.argsort(-dense, kind="stable")[:k]
    idx = np.sort(order).astype(np.uint32)
    return idx, dense[idx].copy()


def _mut_apply_plus(weights, g_idx, g_val, lr):
    out = weights.copy()
    out[g_idx] = out[g_idx] + np.float32(lr) * g_val
    return out


PINS = [pin_apply_update_and_mask, pin_topk_allreduce, pin_dense_topk_and_p2_equals_tree,
        pin_local_select_bruteforce, pin_local_select_library_topk, pin_local_select_invariants,
        pin_local_select_special_k, pin_denormals_not_flushed, pin_merge_dense_definition,
        pin_merge_special_supports, pin_tree_p1_p2, pin_tree_shared_support,
        pin_tree_order_by_composition, pin_tree_not_the_dense_topk, pin_average_is_exact_scale,
        pin_restore_closed_form, pin_hand_worked_example, pin_step_feedback_and_bounds]


@pytest.mark.parametrize("pin", PINS, ids=[p.__name__ for p in PINS])
def test_pin(pin):
    pin()


# --------------------------------------------------------------------------
# planted mistakes: each mutant of the oracle must trip at least one pin
# --------------------------------------------------------------------------

def _mut_tie_high_index(keys, index, k):
    comp = (keys.astype(np.uint64) << np.uint64(32)) | index.astype(np.uint64)
    comp.sort()
    idx = (comp[len(comp) - k:] & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    idx.sort()
    return idx


def _mut_signed_keys(v):
    return np.ascontiguousarray(v, dtype=np.float32).view(np.uint32) ^ np.uint32(0x80000000)


def _mut_accumulate_drops_residual(residual, grad):
    return grad.copy()


def _mut_merge_no_sum(a_idx, a_val, b_idx, b_val, k, _orig=orc.merge):
    keep = ~np.isin(b_idx, a_idx)            # shared indices: b's value is dropped
    pad_idx = np.concatenate([a_idx, b_idx[keep]])
    pad_val = np.concatenate([a_val, b_val[keep]])
    order = np.argsort(pad_idx)
    ui, uv = pad_idx[order].astype(np.uint32), pad_val[order]
    out_idx = orc.first_k_by_magnitude(orc.magnitude_keys(uv), ui, k)
    return out_idx, uv[np.searchsorted(ui, out_idx)].copy()


def _mut_merge_dense_add(a_idx, a_val, b_idx, b_val, k, _orig=orc.merge):
    oi, ov = _orig(a_idx, a_val, b_idx, b_val, k)
    return oi, (ov + f32(0.0)).astype(np.float32)        # -0.0 becomes +0.0


def _mut_tree_chain(loc_idx, loc_val, k, map_fn=map):
    cur = (loc_idx[0], loc_val[0])
    for w in range(1, len(loc_idx)):
        cur = orc.merge(cur[0], cur[1], loc_idx[w], loc_val[w], k)
    return cur[0], (cur[1] / f32(len(loc_idx))).astype(np.float32)


def _mut_tree_no_average(loc_idx, loc_val, k, map_fn=map):
    gi, gs = orc.tree_rounds(loc_idx, loc_val, k)[-1][0]
    return gi.copy(), gs.copy()


def _mut_restore_all(residual, loc_idx, loc_val, g_idx):
    out = residual.copy()
    out[loc_idx] = out[loc_idx] + loc_val
    return out


def _mut_restore_none(residual, loc_idx, loc_val, g_idx):
    return residual.copy()


def _mut_restore_store(residual, loc_idx, loc_val, g_idx):
    out = residual.copy()
    back = ~np.isin(loc_idx, g_idx)
    out[loc_idx[back]] = loc_val[back]                   # store, not add: keeps -0.0
    return out


MUTANTS = [
    ("first_k_by_magnitude", _mut_tie_high_index),
    ("magnitude_keys", _mut_signed_keys),
    ("accumulate", _mut_accumulate_drops_residual),
    ("merge", _mut_merge_no_sum),
    ("merge", _mut_merge_dense_add),
    ("tree", _mut_tree_chain),
    ("tree", _mut_tree_no_average),
    ("residual_restore", _mut_restore_all),
    ("residual_restore", _mut_restore_none),
    ("residual_restore", _mut_restore_store),
    ("apply_update", _mut_apply_plus),
    ("topk_allreduce", _mut_allreduce_reverse_order),
    ("topk_allreduce", _mut_allreduce_no_average),
    ("topk_allreduce", _mut_allreduce_own_twice),
    ("dense_topk", _mut_dense_topk_signed),
]


@pytest.mark.parametrize("name,mutant", MUTANTS, ids=[m[1].__name__ for m in MUTANTS])
def test_planted_mistake_is_caught(monkeypatch, name, mutant):
    monkeypatch.setattr(orc, name, mutant)
    tripped = []
    for pin in PINS:
        try:
            pin()
        except AssertionError:
            tripped.append(pin.__name__)
    assert tripped, f"no pin noticed the planted mistake {mutant.__name__}"


def test_step_through_a_thread_pool_is_the_same_step():
    """`map_fn` only changes who issues the independent calls (workers, pairs of a round),
    never their arithmetic: a thread pool's map must give the bits the builtin map gives."""
    from concurrent.futures import ThreadPoolExecutor
    rng = np.random.default_rng(2024)
    P, m, k = 8, 3000, 40
    res = (rng.standard_normal((P, m)) * 1e-3).astype(np.float32)
    g = (rng.standard_normal((P, m)) * 1e-3).astype(np.float32)
    a = orc.step(res, g, k)
    with ThreadPoolExecutor(max_workers=4) as ex:
        b = orc.step(res, g, k, map_fn=lambda f, it: list(ex.map(f, it)))
    for key in a:
        assert np.array_equal(np.asarray(a[key]).view(np.uint32), np.asarray(b[key]).view(np.uint32)), key
