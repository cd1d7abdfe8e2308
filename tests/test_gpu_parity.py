"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle,
element by element and bit for bit (indices and fp32 values), on the same seeded
inputs.  Sizes here are ones the oracle finishes in seconds; they span several
8192-element blocks, ragged tails, unaligned rows and the degenerate cases."""
import numpy as np
import pytest

from oracle import gtopk_oracle as orc
from paper_1901_04359_amd import workloads as W
from tests.gpu_harness import Device, bits_equal, first_diff, say, to_dev, idx_np, val_np

pytestmark = pytest.mark.gpu


def check_select(dev, res_in, grad, label):
    """Run gtopk_local_select on the device and the oracle on the same rows."""
    P, k = dev.P, dev.k
    dev.set_res(res_in)
    dev.set_grad(grad)
    say(f"local_select {label} P={P} m={dev.m} k={k} stride={dev.stride}")
    gi, gv = dev.local_select()
    gres = dev.residual()
    for w in range(P):
        oi, ov, ores = orc.local_select(res_in[w], grad[w], k)
        assert np.array_equal(gi[w], oi), f"{label} w={w} idx: {first_diff(gi[w], oi)}"
        assert bits_equal(gv[w], ov), f"{label} w={w} val: {first_diff(gv[w], ov)}"
        assert bits_equal(gres[w], ores), f"{label} w={w} residual: {first_diff(gres[w], ores)}"
    return gres


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_local_select_configs_with_feedback(name):
    cfg = W.CONFIGS[name]
    dev = Device(cfg.P, cfg.m, cfg.k)
    res = np.zeros((cfg.P, cfg.m), dtype=np.float32)
    for it in range(cfg.iters):
        g = W.gradients(cfg, it)
        res = check_select(dev, res, g, f"{name} it={it}")


@pytest.mark.parametrize("base,m,P", [("C3", 1_000_003, 2), ("C4a", 2_000_000, 2),
                                      ("C4b", 1_500_001, 2), ("C5", 1_234_567, 2)])
def test_local_select_scaled_recipes(base, m, P):
    cfg = W.scaled(W.CONFIGS[base], m, P=P)
    dev = Device(P, cfg.m, cfg.k)
    res = np.zeros((P, cfg.m), dtype=np.float32)
    for it in range(2):
        g = W.gradients(cfg, it)
        res = check_select(dev, res, g, f"{cfg.name} it={it}")


@pytest.mark.parametrize("m,k,stride", [
    (1, 1, None), (5, 2, None), (5, 5, None), (255, 7, None), (8191, 100, None), (8192, 8192, None),
    (8193, 1, None), (20_001, 333, 20_003),      # odd stride: rows are not 16-byte aligned
    (40_000, 40_000, None), (100_000, 1, None), (65_537, 66, 65_540),
])
def test_local_select_shapes(m, k, stride):
    P = 2
    rng = np.random.default_rng(m * 31 + k)
    dev = Device(P, m, k, stride=stride)
    res = (rng.standard_normal((P, m)) * 1e-3).astype(np.float32)
    grad = (rng.standard_normal((P, m)) * 1e-3).astype(np.float32)
    check_select(dev, res, grad, "shape")


@pytest.mark.parametrize("kind", ["all_equal", "all_zero", "special", "few_levels", "one_spike"])
def test_local_select_degenerate_values(kind):
    P, m, k = 2, 50_000, 777
    rng = np.random.default_rng(1)
    if kind == "all_equal":        # every magnitude ties: the lowest k indices win
        grad = np.where(rng.random((P, m)) < 0.5, -1, 1).astype(np.float32) * np.float32(0.125)
    elif kind == "all_zero":
        grad = np.zeros((P, m), dtype=np.float32)
        grad[:, ::3] = -0.0
    elif kind == "special":
        grad = np.stack([W.special_values(m, seed=s) for s in range(P)])
    elif kind == "few_levels":
        grad = rng.integers(-3, 4, (P, m)).astype(np.float32) * np.float32(0.5)
    else:
        grad = np.zeros((P, m), dtype=np.float32)
        grad[:, 12345] = 7.0
    res = np.zeros((P, m), dtype=np.float32)
    if kind == "special":
        res = np.stack([W.special_values(m, seed=10 + s) for s in range(P)])
    dev = Device(P, m, k)
    check_select(dev, res, grad, kind)


def run_merge(a_idx, a_val, b_idx, b_val, k):
    import torch
    from paper_1901_04359_amd import binding as B
    batch = a_idx.shape[0]
    ws = B.alloc_merge_workspace(k, batch)
    ws.fill_(0x5A)
    out_idx = torch.zeros((batch, k), dtype=torch.int32, device="cuda")
    out_val = torch.zeros((batch, k), dtype=torch.float32, device="cuda")
    B.gtopk_merge(to_dev(a_idx), to_dev(a_val), to_dev(b_idx), to_dev(b_val), k, batch, k,
                  out_idx, out_val, k, ws)
    torch.cuda.synchronize()
    return idx_np(out_idx), val_np(out_val)


@pytest.mark.parametrize("kind", ["gauss", "ties", "cancel"])
@pytest.mark.parametrize("k,m", [(1, 10), (2, 3), (64, 64), (255, 5000), (256, 5000), (257, 5000),
                                 (5000, 200_000), (14_728, 1_000_000), (65_536, 300_000),
                                 (65_537, 300_000), (70_001, 70_001), (131_075, 5_000_000),
                                 (600_001, 5_000_000),
                                 # either side of the sizes at which the union changes kernels
                                 (131_072, 1_000_000), (131_073, 1_000_000),
                                 (524_288, 3_000_000), (524_289, 3_000_000)])
def test_merge_parity(kind, k, m):
    batch = 3
    idx, val = W.ksets(2 * batch, k, m, seed=k, overlap=0.4, value_kind=kind)
    a_idx, a_val = idx[0::2].copy(), val[0::2].copy()
    b_idx, b_val = idx[1::2].copy(), val[1::2].copy()
    say(f"merge kind={kind} k={k} m={m} batch={batch}")
    gi, gv = run_merge(a_idx, a_val, b_idx, b_val, k)
    for b in range(batch):
        oi, ov = orc.merge(a_idx[b], a_val[b], b_idx[b], b_val[b], k)
        assert np.array_equal(gi[b], oi), f"b={b} idx: {first_diff(gi[b], oi)}"
        assert bits_equal(gv[b], ov), f"b={b} val: {first_diff(gv[b], ov)}"


@pytest.mark.parametrize("kind", ["gauss", "ties", "cancel"])
@pytest.mark.parametrize("k,batch", [(300_001, 16), (260_000, 8)])
def test_merge_long_groups(kind, k, batch):
    """Batches whose merged sets are cut into groups of 4096 and 8192 slots, which the select
    walks four slots per load (a batch of three, as above, gets shorter groups); "ties" fills
    the bin of the k-th key far beyond what a block parks in LDS."""
    m = 6_000_000
    idx, val = W.ksets(2 * batch, k, m, seed=k + batch, overlap=0.4, value_kind=kind)
    a_idx, a_val = idx[0::2].copy(), val[0::2].copy()
    b_idx, b_val = idx[1::2].copy(), val[1::2].copy()
    say(f"merge, long groups: kind={kind} k={k} m={m} batch={batch}")
    gi, gv = run_merge(a_idx, a_val, b_idx, b_val, k)
    for b in range(batch):
        oi, ov = orc.merge(a_idx[b], a_val[b], b_idx[b], b_val[b], k)
        assert np.array_equal(gi[b], oi), f"b={b} idx: {first_diff(gi[b], oi)}"
        assert bits_equal(gv[b], ov), f"b={b} val: {first_diff(gv[b], ov)}"


def _gap_ksets(n_sets, k, m, seed):
    """Index sets for very large k without a permutation of [0, m): ascending random gaps."""
    rng = np.random.default_rng(seed)
    idx = np.empty((n_sets, k), dtype=np.uint32)
    val = np.empty((n_sets, k), dtype=np.float32)
    for s in range(n_sets):
        gaps = rng.integers(1, 2 * (m // k), k, dtype=np.int64)       # mean m / k
        pos = np.cumsum(gaps) - 1
        assert pos[-1] < m
        idx[s] = pos.astype(np.uint32)
        val[s] = rng.standard_normal(k).astype(np.float32)
    return idx, val


def _shared_ksets(rng, k, m, shared, kind):
    """One pair of ascending index sets of k entries in [0, m) of which `shared` indices are common,
    with values of one kind: "gauss"; "ties" (five magnitudes, both signs); "cancel" (opposite
    values at the shared indices); "plateau" (every magnitude below a random quantile is raised
    to it, so the k-th key of the merge lies among up to millions of equal keys)."""
    n = 2 * k - shared
    cand = np.flatnonzero(rng.random(m) < min(1.0, 1.03 * n / m + 1e-3))
    while cand.size < n:
        cand = np.flatnonzero(rng.random(m) < min(1.0, 1.2 * n / m + 1e-2))
    pool = np.sort(cand[rng.permutation(cand.size)[:n]])
    who = np.empty(n, dtype=np.int8)
    perm = rng.permutation(n)
    who[perm[:k - shared]] = 1
    who[perm[k - shared:2 * (k - shared)]] = 2
    who[perm[2 * (k - shared):]] = 3
    ia, ib = pool[(who & 1) != 0].astype(np.uint32), pool[(who & 2) != 0].astype(np.uint32)

    def values():
        v = rng.standard_normal(k).astype(np.float32)
        if kind == "ties":
            levels = np.array([0.125, 0.25, 0.5, 1.0, 2.0], dtype=np.float32)
            v = np.copysign(rng.choice(levels, k), v).astype(np.float32)
        elif kind == "plateau":
            c = np.float32(np.quantile(np.abs(v), rng.uniform(0.3, 0.8)))
            v = np.where(np.abs(v) < c, np.copysign(c, v), v).astype(np.float32)
        return v
    va, vb = values(), values()
    if kind == "cancel":
        vb[np.isin(ib, ia)] = -va[np.isin(ia, ib)]
    return ia, va, ib, vb


@pytest.mark.parametrize("k,spread,batch,kind,shared", [
    (530_001, 1.3, 3, "plateau", 0.1), (1_048_577, 2.0, 2, "ties", 0.5),
    (1_700_003, 3.0, 2, "cancel", 0.9), (2_500_000, 1.5, 1, "gauss", 1.0),
    # either side of the size from which a merge goes through a sampled threshold
    (4_194_304, 1.2, 1, "plateau", 0.0), (4_194_305, 1.2, 2, "plateau", 0.5),
    (5_000_001, 2.5, 1, "ties", 0.5), (4_700_000, 4.0, 2, "cancel", 0.1)])
def test_merge_very_large_sets(k, spread, batch, kind, shared):
    """Merged sets of more than 2^20 slots: their select keeps the keys of the k-th key's bin
    with their groups and finishes once per set; with more than 2^22 entries per operand the
    union is filtered first.  Ties and plateaus fill that bin far beyond what the finish holds
    in LDS."""
    import torch
    from paper_1901_04359_amd import binding as B
    m = int(2 * k * spread)
    rng = np.random.default_rng(k + batch)
    sets = [_shared_ksets(rng, k, m, int(round(shared * k)), kind) for _ in range(batch)]
    a_idx, a_val, b_idx, b_val = (np.stack([s[j] for s in sets]) for j in range(4))
    assert B.gtopk_debug_plan(m, k, 2)["merge_filtered"] == (1 if k > 1 << 22 else 0)
    say(f"merge, very large sets: k={k} m={m} batch={batch} kind={kind} shared={shared}")
    ws = B.alloc_merge_workspace(k, batch)
    ws.fill_(0x5A)
    out_idx = torch.zeros((batch, k), dtype=torch.int32, device="cuda")
    out_val = torch.zeros((batch, k), dtype=torch.float32, device="cuda")
    B.gtopk_merge(to_dev(a_idx), to_dev(a_val), to_dev(b_idx), to_dev(b_val), k, batch, k, out_idx, out_val, k, ws)
    gi, gv = idx_np(out_idx), val_np(out_val)
    for b in range(batch):
        oi, ov = orc.merge(a_idx[b], a_val[b], b_idx[b], b_val[b], k)
        assert np.array_equal(gi[b], oi), f"b={b} idx: {first_diff(gi[b], oi)}"
        assert bits_equal(gv[b], ov), f"b={b} val: {first_diff(gv[b], ov)}"


@pytest.mark.parametrize("P,k,kind,shared", [(8, 700_001, "plateau", 0.3), (4, 1_300_000, "ties", 0.9)])
def test_tree_very_large_sets(P, k, kind, shared):
    """Every round of these trees selects from merged sets of more than 2^20 slots."""
    m = 5 * k
    rng = np.random.default_rng(P + k)
    idx = np.empty((P, k), dtype=np.uint32)
    val = np.empty((P, k), dtype=np.float32)
    for p in range(0, P, 2):
        idx[p], val[p], idx[p + 1], val[p + 1] = _shared_ksets(rng, k, m, int(round(shared * k)), kind)
    dev = Device(P, k, k)
    dev.loc_idx.copy_(to_dev(idx))
    dev.loc_val.copy_(to_dev(val))
    say(f"tree of very large sets P={P} k={k} m={m} kind={kind}")
    gi, gv = dev.tree()
    oi, ov = orc.tree(list(idx), list(val), k)
    assert np.array_equal(gi, oi), first_diff(gi, oi)
    assert bits_equal(gv, ov), first_diff(gv, ov)


def test_merge_speculative_threshold_hits_and_misses():
    """Merges of more than 2^22 entries keep only the slots of the union that reach a threshold
    taken from a sample.  Pair 0 is ordinary; pair 1 has its large values exactly where the
    sample looks in both operands, so the threshold lands among them and fewer than k slots are
    kept: that pair is merged once more from its complete union; pair 2 is all ties (and the
    operands cancel at every shared index).  All in one launch, bit for bit against the oracle."""
    import torch
    from paper_1901_04359_amd import binding as B
    k, m, batch = 4_200_003, 33_554_432, 3
    plan = B.gtopk_debug_plan(m, k, 2)
    assert plan["merge_filtered"] == 1
    idx, val = _gap_ksets(2 * batch, k, m, seed=77)
    a_idx, a_val = idx[0::2].copy(), val[0::2].copy()
    b_idx, b_val = idx[1::2].copy(), val[1::2].copy()
    assert np.isin(b_idx[0][:100_000], a_idx[0]).sum() > 1000          # the operands do share indices
    rng = np.random.default_rng(5)
    t = np.arange(plan["merge_n_tiles"], dtype=np.int64)[:, None] * plan["merge_tile_stride"]
    pos = (t + np.arange(plan["tile_len"], dtype=np.int64)[None, :]).ravel()
    pos = pos[pos < k]
    assert 2 * pos.size < k
    a_val[1] *= np.float32(1e-3)
    b_val[1] *= np.float32(1e-3)
    a_val[1, pos] = (1.0 + rng.random(pos.size)).astype(np.float32)
    b_val[1, pos] = -(1.0 + rng.random(pos.size)).astype(np.float32)
    a_val[2] = np.float32(0.25)
    b_val[2] = np.float32(-0.25)
    say(f"merge through a speculative threshold k={k} batch={batch}")
    ws = B.alloc_merge_workspace(k, batch)
    ws.fill_(0x5A)
    out_idx = torch.zeros((batch, k), dtype=torch.int32, device="cuda")
    out_val = torch.zeros((batch, k), dtype=torch.float32, device="cuda")
    B.gtopk_merge(to_dev(a_idx), to_dev(a_val), to_dev(b_idx), to_dev(b_val), k, batch, k, out_idx, out_val, k, ws)
    kept = B.gtopk_debug_merge_kept(ws, k, batch)
    assert kept[0] >= k and kept[1] < k, kept
    gi, gv = idx_np(out_idx), val_np(out_val)
    for b in range(batch):
        oi, ov = orc.merge(a_idx[b], a_val[b], b_idx[b], b_val[b], k)
        assert np.array_equal(gi[b], oi), f"b={b} (kept {kept[b]}) idx: {first_diff(gi[b], oi)}"
        assert bits_equal(gv[b], ov), f"b={b} (kept {kept[b]}) val: {first_diff(gv[b], ov)}"


@pytest.mark.parametrize("layout", ["a_below_b", "b_below_a", "identical", "interleaved",
                                    "blocks", "one_shared"])
@pytest.mark.parametrize("k", [300, 66_000, 100_003])
def test_merge_structured_index_sets(layout, k):
    """Index layouts that put the cut points of the union at their extremes."""
    rng = np.random.default_rng(k)
    t = np.arange(k, dtype=np.uint32)
    if layout == "a_below_b":
        a_idx, b_idx = t, t + k
    elif layout == "b_below_a":
        a_idx, b_idx = t + k + 5, t
    elif layout == "identical":
        a_idx, b_idx = 3 * t, 3 * t
    elif layout == "interleaved":
        a_idx, b_idx = 2 * t, 2 * t + 1
    elif layout == "blocks":          # long runs of A, then of B, some of them shared
        blk, off = t // 5000, t % 5000
        a_idx = blk * 20_000 + 10_000 + off
        b_idx = blk * 20_000 + off + np.choose(blk % 3, [10_000, 0, 15_000])
    else:
        a_idx, b_idx = 2 * t, 2 * t + 1
        b_idx = b_idx.copy()
        b_idx[k // 2] = a_idx[k // 2]
    a_idx = np.ascontiguousarray(a_idx, dtype=np.uint32)[None]
    b_idx = np.ascontiguousarray(b_idx, dtype=np.uint32)[None]
    a_val = rng.standard_normal((1, k)).astype(np.float32)
    b_val = rng.standard_normal((1, k)).astype(np.float32)
    say(f"merge layout={layout} k={k}")
    gi, gv = run_merge(a_idx, a_val, b_idx, b_val, k)
    oi, ov = orc.merge(a_idx[0], a_val[0], b_idx[0], b_val[0], k)
    assert np.array_equal(gi[0], oi), first_diff(gi[0], oi)
    assert bits_equal(gv[0], ov), first_diff(gv[0], ov)


@pytest.mark.parametrize("P", [1, 2, 4, 8, 16, 32])
@pytest.mark.parametrize("k,m,kind", [(66, 65_536, "gauss"), (1000, 30_000, "cancel"),
                                      (300, 2000, "ties")])
def test_tree_parity(P, k, m, kind):
    idx, val = W.ksets(P, k, m, seed=P + k, overlap=0.5, value_kind=kind)
    dev = Device(P, k, k)          # only the k-set buffers and the workspace are used
    dev.loc_idx.copy_(to_dev(idx))
    dev.loc_val.copy_(to_dev(val))
    say(f"tree P={P} k={k} m={m} kind={kind}")
    gi, gv = dev.tree()
    oi, ov = orc.tree(list(idx), list(val), k)
    assert np.array_equal(gi, oi), first_diff(gi, oi)
    assert bits_equal(gv, ov), first_diff(gv, ov)


@pytest.mark.parametrize("kind", ["gauss", "ties"])
def test_tree_large_sets(kind):
    """A tree of 16 sets of 300,000 entries: unions cut by output position, and rounds whose
    merged sets are cut into groups of 4864, 2560, 1280 and 768 slots (the select walks the
    first round's four slots per load, the others slot by slot)."""
    P, k, m = 16, 300_000, 6_000_000
    idx, val = W.ksets(P, k, m, seed=P + k, overlap=0.5, value_kind=kind)
    dev = Device(P, k, k)
    dev.loc_idx.copy_(to_dev(idx))
    dev.loc_val.copy_(to_dev(val))
    say(f"tree of large sets P={P} k={k} m={m} kind={kind}")
    gi, gv = dev.tree()
    oi, ov = orc.tree(list(idx), list(val), k)
    assert np.array_equal(gi, oi), first_diff(gi, oi)
    assert bits_equal(gv, ov), first_diff(gv, ov)


def test_tree_every_round_matches_oracle():
    """Intermediate sets of every round, through gtopk_merge, in the tree's pairing."""
    P, k, m = 8, 500, 20_000
    idx, val = W.ksets(P, k, m, seed=77, overlap=0.6, value_kind="cancel")
    hist = orc.tree_rounds(list(idx), list(val), k)
    cur_i, cur_v = idx.copy(), val.copy()
    for j, rnd in enumerate(hist):
        say(f"tree round {j}")
        gi, gv = run_merge(cur_i[0::2].copy(), cur_v[0::2].copy(),
                           cur_i[1::2].copy(), cur_v[1::2].copy(), k)
        survivors = [c for c in rnd if c is not None]
        assert len(survivors) == gi.shape[0]
        for p, (oi, ov) in enumerate(survivors):
            assert np.array_equal(gi[p], oi) and bits_equal(gv[p], ov), f"round {j} pair {p}"
        cur_i, cur_v = gi, gv


@pytest.mark.parametrize("P,m,k", [(4, 65_536, 66), (2, 1000, 1000), (8, 100_000, 5000)])
def test_restore_parity(P, m, k):
    rng = np.random.default_rng(P * m + k)
    res = (rng.standard_normal((P, m))).astype(np.float32)
    loc_idx, loc_val = W.ksets(P, k, m, seed=5, overlap=0.5)
    loc_val[:, ::7] = -0.0
    for w in range(P):
        res[w, loc_idx[w]] = 0.0
    g_idx = np.sort(rng.choice(m, k, replace=False)).astype(np.uint32)
    g_idx[: k // 2] = np.sort(loc_idx[0][: k // 2])       # make some local entries survive
    g_idx = np.unique(g_idx)
    while g_idx.size < k:
        extra = rng.choice(m, k - g_idx.size, replace=False).astype(np.uint32)
        g_idx = np.unique(np.concatenate([g_idx, extra]))
    g_idx = g_idx[:k]
    dev = Device(P, m, k)
    dev.set_res(res)
    dev.loc_idx.copy_(to_dev(loc_idx))
    dev.loc_val.copy_(to_dev(loc_val))
    dev.g_idx.copy_(to_dev(g_idx))
    say(f"restore P={P} m={m} k={k}")
    dev.restore()
    out = dev.residual()
    for w in range(P):
        exp = orc.residual_restore(res[w], loc_idx[w], loc_val[w], g_idx)
        assert bits_equal(out[w], exp), f"w={w}: {first_diff(out[w], exp)}"


def check_steps(cfg, grads_of_iter, iters, label, want_loc=True, general=False):
    """`general`: go through gtopk_step_carry, which always takes the general kernels (small
    problems otherwise take gtopk_step's few-launch path)."""
    P, m, k = cfg.P, cfg.m, cfg.k
    dev = Device(P, m, k)
    res = np.zeros((P, m), dtype=np.float32)
    dev.set_res(res)
    for it in range(iters):
        g = grads_of_iter(it)
        dev.set_grad(g)
        say(f"step {label} it={it} P={P} m={m} k={k} general={general}")
        gi, gv = dev.step_carry(want_loc=want_loc) if general else dev.step(want_loc=want_loc)
        exp = orc.step(res, g, k)
        if want_loc:
            li, lv = idx_np(dev.loc_idx), val_np(dev.loc_val)
            assert np.array_equal(li, exp["loc_idx"]), f"it={it} loc_idx {first_diff(li, exp['loc_idx'])}"
            assert bits_equal(lv, exp["loc_val"]), f"it={it} loc_val {first_diff(lv, exp['loc_val'])}"
        assert np.array_equal(gi, exp["g_idx"]), f"it={it} g_idx {first_diff(gi, exp['g_idx'])}"
        assert bits_equal(gv, exp["g_val"]), f"it={it} g_val {first_diff(gv, exp['g_val'])}"
        out = dev.residual()
        assert bits_equal(out, exp["residual"]), f"it={it} residual {first_diff(out, exp['residual'])}"
        res = exp["residual"]


@pytest.mark.parametrize("general", [False, True])
@pytest.mark.parametrize("name", ["C1", "C2"])
def test_step_configs_all_iterations(name, general):
    from paper_1901_04359_amd import binding as B
    cfg = W.CONFIGS[name]
    assert B.gtopk_debug_plan(cfg.m, cfg.k, cfg.P)["small_path"] == 1     # the two small configs
    check_steps(cfg, lambda it: W.gradients(cfg, it), cfg.iters, name, general=general)


@pytest.mark.parametrize("base,m,P", [("C3", 500_009, 16), ("C4a", 1_000_000, 32),
                                      ("C4b", 300_000, 32), ("C5", 400_001, 32)])
def test_step_scaled_recipes(base, m, P):
    cfg = W.scaled(W.CONFIGS[base], m, P=P)
    check_steps(cfg, lambda it: W.gradients(cfg, it), 3, cfg.name, want_loc=(base != "C4b"))


def test_step_correlated_workers():
    """Workers share a component, so merges meet matching indices in every round."""
    cfg = W.scaled(W.CONFIGS["C2"], 200_003, k=2000, P=8, name="correlated")
    check_steps(cfg, lambda it: W.correlated_gradients(cfg.m, cfg.P, it), 3, "correlated")


def check_carry_steps(cfg, iters, label, event=None):
    """gtopk_step_carry over `iters` iterations against the oracle.  `event(it, modes)` may
    return (gradient scale, wipe residual) for an iteration.  Returns, per iteration, the
    carry modes BEFORE the call (2 = that call skipped sampling), the candidate counts the
    pass left, the list capacity and what `event` asked for."""
    from paper_1901_04359_amd import binding as B
    P, m, k = cfg.P, cfg.m, cfg.k
    dev = Device(P, m, k)
    res = np.zeros((P, m), dtype=np.float32)
    dev.set_res(res)
    trace = []
    for it in range(iters):
        modes = dev.carry_modes()
        scale, wipe = event(it, modes) if event else (1.0, False)
        g = W.gradients(cfg, it)
        if scale != 1.0:
            g = (g * np.float32(scale)).astype(np.float32)
        if wipe:
            res = np.zeros_like(res)
            dev.set_res(res)
        dev.set_grad(g)
        say(f"step_carry {label} it={it} P={P} m={m} k={k} modes={modes} scale={scale} wipe={wipe}")
        gi, gv = dev.step_carry()
        counts, cap = B.gtopk_debug_candidate_counts(dev.ws, m, k, P)
        exp = orc.step(res, g, k)
        li, lv = idx_np(dev.loc_idx), val_np(dev.loc_val)
        assert np.array_equal(li, exp["loc_idx"]), f"it={it} loc_idx {first_diff(li, exp['loc_idx'])}"
        assert bits_equal(lv, exp["loc_val"]), f"it={it} loc_val {first_diff(lv, exp['loc_val'])}"
        assert np.array_equal(gi, exp["g_idx"]), f"it={it} g_idx {first_diff(gi, exp['g_idx'])}"
        assert bits_equal(gv, exp["g_val"]), f"it={it} g_val {first_diff(gv, exp['g_val'])}"
        out = dev.residual()
        assert bits_equal(out, exp["residual"]), f"it={it} residual {first_diff(out, exp['residual'])}"
        res = exp["residual"]
        trace.append((modes, counts, cap, (scale, wipe)))
    return trace


@pytest.mark.parametrize("base,m,P", [("C4a", 1_000_000, 8), ("C4b", 600_000, 4), ("C5", 800_001, 4)])
def test_step_carry_matches_oracle_and_skips_sampling(base, m, P):
    """Thresholds carried from call to call: every iteration bit-exact, and once the k-th
    magnitudes move predictably the calls stop sampling while the pass still keeps between
    k and the list's capacity of candidates."""
    cfg = W.scaled(W.CONFIGS[base], m, P=P)
    trace = check_carry_steps(cfg, 14, cfg.name)
    assert trace[0][0] == [0] * P                       # the first call samples
    skipped = [it for it, t in enumerate(trace) if all(md == 2 for md in t[0])]
    assert len(skipped) >= 3, [t[0] for t in trace]     # the later calls do not
    for it in skipped:
        _, counts, cap, _ = trace[it]
        assert all(cfg.k <= c <= cap for c in counts), (it, counts, cap, cfg.k)


def test_step_carry_survives_jumps_of_the_magnitudes():
    """A carried threshold that has become worthless costs time, never correctness.  Once the
    calls have stopped sampling, the residual is wiped and the gradients shrunk (the k-th
    magnitude drops by far: the pass comes back with fewer than k candidates); later the
    gradients grow a thousand-fold (more candidates than the list holds).  The results stay
    the oracle's and the call after each jump samples again."""
    cfg = W.scaled(W.CONFIGS["C4a"], 700_001, P=4)
    k = cfg.k
    done = {"down": None, "up": None}

    def event(it, modes):
        trusted = all(md == 2 for md in modes)
        if done["down"] is None and it >= 4 and trusted:
            done["down"] = it
            return 0.02, True
        if done["down"] is not None and done["up"] is None and it >= done["down"] + 3 and trusted:
            done["up"] = it
            return 1000.0, False
        return 1.0, False

    trace = check_carry_steps(cfg, 24, "jumps", event)
    assert done["down"] is not None and done["up"] is not None, (done, [t[0] for t in trace])
    d, u = done["down"], done["up"]
    assert all(c < k for c in trace[d][1]), (trace[d][1], k)            # came back short
    assert all(md != 2 for md in trace[d + 1][0])                        # so the next call sampled
    assert all(c > trace[u][2] for c in trace[u][1]), (trace[u][1], trace[u][2])   # overflowed
    if u + 1 < len(trace):
        assert all(md != 2 for md in trace[u + 1][0])


def test_step_is_deterministic():
    cfg = W.scaled(W.CONFIGS["C4a"], 700_001, P=8)
    g = W.gradients(cfg, 0)
    outs = []
    for rep in range(2):
        dev = Device(cfg.P, cfg.m, cfg.k)
        dev.set_grad(g)
        say(f"determinism rep={rep}")
        gi, gv = dev.step()
        outs.append((gi.copy(), gv.copy(), dev.residual().copy(), idx_np(dev.loc_idx).copy()))
    assert np.array_equal(outs[0][0], outs[1][0]) and bits_equal(outs[0][1], outs[1][1])
    assert bits_equal(outs[0][2], outs[1][2]) and np.array_equal(outs[0][3], outs[1][3])


def test_candidate_path_is_the_one_exercised():
    """On the configs' recipes every worker must be served from its candidate list (the
    fast path); on an all-equal-magnitude input the candidates overflow and the dense
    row is read instead (the exact fallback).  Both were checked bit for bit above; this
    test pins WHICH path ran."""
    from paper_1901_04359_amd import binding as B
    for base, m, P in (("C2", 269_722, 8), ("C4a", 2_000_000, 4), ("C4b", 1_000_000, 4),
                       ("C3", 1_000_000, 4), ("C5", 1_500_000, 4)):
        cfg = W.scaled(W.CONFIGS[base], m, P=P)
        dev = Device(P, cfg.m, cfg.k)
        dev.set_grad(W.gradients(cfg, 0))
        say(f"path check {cfg.name}")
        dev.local_select()
        counts, cap = B.gtopk_debug_candidate_counts(dev.ws, cfg.m, cfg.k, P)
        assert all(cfg.k <= c <= cap for c in counts), (cfg.name, counts, cap, cfg.k)
        assert max(counts) <= 2.5 * cfg.k + 4096, (cfg.name, counts, cfg.k)
    P, m, k = 2, 50_000, 777
    dev = Device(P, m, k)
    dev.set_grad(np.full((P, m), 0.125, dtype=np.float32))
    say("path check all-equal")
    dev.local_select()
    counts, cap = B.gtopk_debug_candidate_counts(dev.ws, m, k, P)
    assert all(c > cap for c in counts), (counts, cap)


@pytest.mark.parametrize("m,k,copies", [(1000, 1000, 1), (65_536, 66, 4), (2_000_003, 20_000, 2)])
def test_apply_update_and_dense_mask(m, k, copies):
    import torch
    from paper_1901_04359_amd import binding as B
    rng = np.random.default_rng(m + k)
    Wt = rng.standard_normal((copies, m)).astype(np.float32)
    g_idx = np.sort(rng.choice(m, k, replace=False)).astype(np.uint32)
    g_val = (rng.standard_normal(k) * 1e-3).astype(np.float32)
    g_val[::11] = 0.0
    d_w = to_dev(Wt)
    say(f"apply_update m={m} k={k} copies={copies}")
    for lr in (0.1, 0.01):
        B.gtopk_apply_update(d_w, k, to_dev(g_idx), to_dev(g_val), lr)
        torch.cuda.synchronize()
        for c in range(copies):
            Wt[c] = orc.apply_update(Wt[c], g_idx, g_val, lr)
        out = d_w.cpu().numpy()
        assert bits_equal(out, Wt), first_diff(out, Wt)
    mask = torch.full((m,), 7, dtype=torch.uint8, device="cuda")
    B.gtopk_dense_mask(to_dev(g_idx), k, mask)
    torch.cuda.synchronize()
    assert np.array_equal(mask.cpu().numpy(), orc.dense_mask(g_idx, m))


@pytest.mark.parametrize("rho,m", [(0.25, 1_000_003), (0.0725, 1_000_003), (0.015, 1_000_003),
                                   (0.005, 1_000_003), (0.004, 1_000_003), (0.0005, 1_000_003),
                                   (0.25, 3_000_017)])     # sets of more than 2^20 slots
def test_step_density_schedule(rho, m):
    """The densities of the paper's warm-up schedule (Section IV-B: 0.25, 0.0725, 0.015,
    0.004), the LSTM density 0.005 and the smallest density of its sensitivity study."""
    P = 4
    cfg = W.scaled(W.CONFIGS["C4a"], m, k=max(1, int(round(rho * m))), P=P, name=f"rho={rho}")
    check_steps(cfg, lambda it: W.gradients(cfg, it), 2, cfg.name)
    from paper_1901_04359_amd import binding as B
    dev = Device(P, cfg.m, cfg.k)
    dev.set_grad(W.gradients(cfg, 0))
    dev.local_select()
    counts, cap = B.gtopk_debug_candidate_counts(dev.ws, cfg.m, cfg.k, P)
    assert all(cfg.k <= c <= cap for c in counts), (rho, counts, cap, cfg.k)


@pytest.mark.parametrize("P,m,k,stride", [
    (1, 100_000, 100, None),          # P = 1: no tree round, g = loc / 1
    (2, 5_000, 5_000, None),          # k = m: everything is selected everywhere
    (4, 32_768, 33, None),            # exactly one streaming block per worker
    (4, 32_769, 33, 32_771),          # one element into a second block; rows not 16-byte aligned
    (8, 131_071, 1, None),            # k = 1
    (64, 40_000, 40, None),           # more workers than the configs use (six rounds)
    (256, 5_000, 50, None),           # eight rounds, 128 pairs in the first
    (4, 300_001, 3_000, 300_005),     # padded rows, odd stride
])
@pytest.mark.parametrize("general", [False, True])
def test_step_shapes(P, m, k, stride, general):
    rng = np.random.default_rng(P * 7 + m + k)
    dev = Device(P, m, k, stride=stride)
    res = np.zeros((P, m), dtype=np.float32)
    dev.set_res(res)
    for it in range(2):
        g = (rng.standard_normal((P, m)) * 1e-3).astype(np.float32)
        dev.set_grad(g)
        say(f"step shapes P={P} m={m} k={k} stride={stride} it={it} general={general}")
        gi, gv = dev.step_carry() if general else dev.step()
        exp = orc.step(res, g, k)
        assert np.array_equal(idx_np(dev.loc_idx), exp["loc_idx"])
        assert bits_equal(val_np(dev.loc_val), exp["loc_val"])
        assert np.array_equal(gi, exp["g_idx"]) and bits_equal(gv, exp["g_val"])
        out = dev.residual()
        assert bits_equal(out, exp["residual"]), first_diff(out, exp["residual"])
        res = exp["residual"]
    if stride is not None:      # the padding between rows must be untouched
        pad = dev.res_buf[: P * stride].view(P, stride)[:, m:].cpu().numpy()
        assert not pad.any()


@pytest.mark.parametrize("kind", ["all_equal", "all_zero", "special", "few_levels", "one_spike", "under"])
@pytest.mark.parametrize("P,m,k", [(4, 65_536, 66), (8, 300_000, 300), (64, 9_000, 64),
                                   (8, 1_048_573, 512), (2, 700, 512)])
def test_small_path_degenerate_rows_and_limits(kind, P, m, k):
    """gtopk_step's few-launch path (one block per worker, one block for the tree) at the
    limits of the sizes it takes, on rows that make a worker fall back to its dense row
    inside that block, next to ordinary workers."""
    from paper_1901_04359_amd import binding as B
    plan = B.gtopk_debug_plan(m, k, P)
    assert plan["small_path"] == 1
    rng = np.random.default_rng(P + m + k)
    g = (rng.standard_normal((P, m)) * 1e-3).astype(np.float32)
    for w in range(0, P, 2):                  # every other worker is a special row
        if kind == "all_equal":
            g[w] = np.where(rng.random(m) < 0.5, -1, 1).astype(np.float32) * np.float32(0.125)
        elif kind == "all_zero":
            g[w] = 0.0
            g[w, ::3] = -0.0
        elif kind == "special":
            g[w] = W.special_values(m, seed=w)
        elif kind == "few_levels":
            g[w] = rng.integers(-1, 2, m).astype(np.float32) * np.float32(0.5)
        elif kind == "one_spike":
            g[w] = 0.0
            g[w, m // 3] = 7.0
        else:                                  # large magnitudes only where the sampler looks
            t = np.arange(plan["small_n_tiles"], dtype=np.int64)[:, None] * plan["small_tile_stride"]
            pos = (t + np.arange(plan["tile_len"], dtype=np.int64)[None, :]).ravel()
            pos = pos[pos < m]
            if pos.size < m and plan["small_target"] < k - 1:
                at = rng.choice(pos, min(pos.size, k - 1), replace=False)
                g[w, at] = (1.0 + rng.random(at.size)).astype(np.float32)
    dev = Device(P, m, k)
    res = np.zeros((P, m), dtype=np.float32)
    dev.set_res(res)
    for it in range(2):
        dev.set_grad(g)
        say(f"small path kind={kind} P={P} m={m} k={k} it={it}")
        gi, gv = dev.step()
        exp = orc.step(res, g, k)
        assert np.array_equal(idx_np(dev.loc_idx), exp["loc_idx"]), first_diff(idx_np(dev.loc_idx), exp["loc_idx"])
        assert bits_equal(val_np(dev.loc_val), exp["loc_val"])
        assert np.array_equal(gi, exp["g_idx"]), first_diff(gi, exp["g_idx"])
        assert bits_equal(gv, exp["g_val"]), first_diff(gv, exp["g_val"])
        out = dev.residual()
        assert bits_equal(out, exp["residual"]), first_diff(out, exp["residual"])
        res = exp["residual"]
        g = (rng.standard_normal((P, m)) * 1e-3).astype(np.float32)     # then ordinary gradients


def test_step_matches_the_three_calls():
    """gtopk_step (which fuses zeroing and restore) against gtopk_local_select + gtopk_tree +
    gtopk_residual_restore on the same inputs, including -0.0 entries that get selected."""
    P, m, k = 4, 50_000, 30_000            # k so large that zeros and -0.0 are selected
    rng = np.random.default_rng(99)
    g = (rng.standard_normal((P, m)) * 1e-3).astype(np.float32)
    g[:, ::2] = 0.0
    g[:, ::6] = -0.0
    a = Device(P, m, k)
    b = Device(P, m, k)
    for dev in (a, b):
        dev.set_grad(g)
    say("step vs three calls")
    gi_a, gv_a = a.step()
    b.local_select()
    gi_b, gv_b = b.tree()
    b.restore()
    assert np.array_equal(gi_a, gi_b) and bits_equal(gv_a, gv_b)
    assert np.array_equal(idx_np(a.loc_idx), idx_np(b.loc_idx))
    assert bits_equal(val_np(a.loc_val), val_np(b.loc_val))
    assert bits_equal(a.residual(), b.residual()), first_diff(a.residual(), b.residual())
    exp = orc.step(np.zeros((P, m), dtype=np.float32), g, k)
    assert bits_equal(a.residual(), exp["residual"])


# --------------------------------------------------------------------------
# the two comparison aggregations: Algorithm 1's TopKAllReduce, Algorithm 2's second top-k
# --------------------------------------------------------------------------

def run_allreduce(idx, val, m):
    import torch
    from paper_1901_04359_amd import binding as B
    P, k = idx.shape
    dense = torch.full((m,), float("nan"), dtype=torch.float32, device="cuda")   # every element must be written
    ws = B.alloc_allreduce_workspace(m, P)
    ws.fill_(0xA5)
    B.gtopk_topk_allreduce(to_dev(idx), to_dev(val), P, k, dense, ws)
    return dense


@pytest.mark.parametrize("P,k,m,kind,overlap", [
    (1, 10, 100, "gauss", 0.0), (2, 17, 200, "cancel", 0.9), (3, 300, 2000, "ties", 0.5),
    (4, 66, 65_536, "gauss", 0.3), (8, 5000, 8192, "gauss", 0.9),       # one range, long slices
    (5, 8193, 8193, "gauss", 1.0),                                      # k = m: everything everywhere
    (32, 1000, 1_000_003, "cancel", 0.5), (16, 20_000, 300_001, "gauss", 0.7),
    (100, 50, 40_000, "gauss", 0.2),
])
def test_topk_allreduce_parity(P, k, m, kind, overlap):
    idx, val = W.ksets(P, k, m, seed=P * 1000 + k, overlap=overlap, value_kind=kind)
    say(f"topk_allreduce P={P} k={k} m={m} kind={kind}")
    dense = run_allreduce(idx, val, m).cpu().numpy()
    exp = orc.topk_allreduce(list(idx), list(val), m)
    assert bits_equal(dense, exp), first_diff(dense, exp)


def test_topk_allreduce_order_and_signed_zero():
    """Adds at one index happen in rank order; a lone -0.0 comes out as +0.0."""
    m = 20_000
    idx = np.array([[5, 9000], [5, 9001], [5, 9002], [6, 19_999]], dtype=np.uint32)
    val = np.array([[1.0, -0.0], [1e8, 2.0], [-1e8, 3.0], [8.0, -0.0]], dtype=np.float32)
    say("topk_allreduce order")
    dense = run_allreduce(idx, val, m).cpu().numpy()
    exp = orc.topk_allreduce(list(idx), list(val), m)
    assert bits_equal(dense, exp), first_diff(dense, exp)
    assert dense[5] == 0.0 and dense[6] == 2.0
    assert dense[[9000, 19_999]].view(np.uint32).tolist() == [0, 0]


@pytest.mark.parametrize("m,k,kind", [
    (100, 10, "gauss"), (5000, 5000, "gauss"), (70_000, 1, "gauss"), (300_001, 3000, "ties"),
    (1_000_003, 1000, "sparse"), (1_000_003, 50_000, "sparse"), (2_500_000, 2500, "gauss"),
])
def test_dense_topk_parity(m, k, kind):
    import torch
    from paper_1901_04359_amd import binding as B
    rng = np.random.default_rng(m + k)
    if kind == "gauss":
        d = rng.standard_normal(m).astype(np.float32)
    elif kind == "ties":
        d = (rng.integers(-3, 4, m)).astype(np.float32) * np.float32(0.5)
    else:                      # what an allreduce of sparse sets leaves: mostly +0.0
        d = np.zeros(m, dtype=np.float32)
        at = rng.choice(m, min(m, 3 * k // 2), replace=False)
        d[at] = rng.standard_normal(at.shape[0]).astype(np.float32)
    dd = to_dev(d)
    g_idx = torch.zeros(k, dtype=torch.int32, device="cuda")
    g_val = torch.zeros(k, dtype=torch.float32, device="cuda")
    ws = B.alloc_workspace(m, k, 1)
    ws.fill_(0xA5)
    say(f"dense_topk m={m} k={k} kind={kind}")
    B.gtopk_dense_topk(dd, k, g_idx, g_val, ws)
    oi, ov = orc.dense_topk(d, k)
    gi, gv = idx_np(g_idx), val_np(g_val)
    assert np.array_equal(gi, oi), first_diff(gi, oi)
    assert bits_equal(gv, ov), first_diff(gv, ov)
    assert bits_equal(dd.cpu().numpy(), d)          # the input is not modified


def test_naive_gtopk_iteration_matches_oracle():
    """Algorithm 2 lines 4-15 chained through the entry points: local selection, sparse
    all-reduce, second top-k, extra residual, model update."""
    import torch
    from paper_1901_04359_amd import binding as B
    cfg = W.scaled(W.CONFIGS["C2"], 200_003, k=400, P=8, name="naive")
    P, m, k = cfg.P, cfg.m, cfg.k
    dev = Device(P, m, k)
    res = np.zeros((P, m), dtype=np.float32)
    wts = np.linspace(-1, 1, m, dtype=np.float32)
    d_w = to_dev(wts)
    dense = torch.empty(m, dtype=torch.float32, device="cuda")
    ws_ar = B.alloc_allreduce_workspace(m, P)
    ws_1 = B.alloc_workspace(m, k, 1)
    for it in range(2):
        g = W.gradients(cfg, it)
        dev.set_res(res)
        dev.set_grad(g)
        say(f"naive gtopk iteration {it}")
        li, lv = dev.local_select()
        B.gtopk_topk_allreduce(dev.loc_idx, dev.loc_val, P, k, dense, ws_ar)
        B.gtopk_dense_topk(dense, k, dev.g_idx, dev.g_val, ws_1)
        B.gtopk_residual_restore(dev.res, k, dev.loc_idx, dev.loc_val, dev.g_idx)
        B.gtopk_apply_update(d_w, k, dev.g_idx, dev.g_val, 0.05)
        # oracle
        o_li, o_lv, o_res = [], [], []
        for w in range(P):
            a, b, c = orc.local_select(res[w], g[w], k)
            o_li.append(a); o_lv.append(b); o_res.append(c)
        o_dense = orc.topk_allreduce(o_li, o_lv, m)
        o_gi, o_gv = orc.dense_topk(o_dense, k)
        res = np.stack([orc.residual_restore(o_res[w], o_li[w], o_lv[w], o_gi) for w in range(P)])
        wts = orc.apply_update(wts, o_gi, o_gv, 0.05)
        assert np.array_equal(idx_np(dev.g_idx), o_gi)
        assert bits_equal(val_np(dev.g_val), o_gv)
        assert bits_equal(dense.cpu().numpy(), o_dense)
        assert bits_equal(dev.residual(), res)
        assert bits_equal(d_w.cpu().numpy(), wts)


def test_hand_worked_example_on_the_gpu():
    """The pencil-and-paper example of tests/golden (m = 8, P = 4, k = 2) through the library:
    the expected values come from the fixture, not from the oracle."""
    import json
    import os
    import torch
    from paper_1901_04359_amd import binding as B
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "hand_worked_p4_k2.json")
    with open(path) as fh:
        ex = json.load(fh)
    P, m, k = ex["P"], ex["m"], ex["k"]
    dev = Device(P, m, k)
    dev.set_grad(np.array(ex["grad"], dtype=np.float32))
    say("hand-worked example: step")
    gi, gv = dev.step()
    assert idx_np(dev.loc_idx).tolist() == ex["loc_idx"] and val_np(dev.loc_val).tolist() == ex["loc_val"]
    assert gi.tolist() == ex["g_idx"] and gv.tolist() == ex["g_val"]
    assert dev.residual().tolist() == ex["residual"]
    say("hand-worked example: all-reduce, dense top-k, restore")
    dense = torch.empty(m, dtype=torch.float32, device="cuda")
    B.gtopk_topk_allreduce(dev.loc_idx, dev.loc_val, P, k, dense, B.alloc_allreduce_workspace(m, P))
    assert dense.cpu().numpy().tolist() == ex["alg1_dense"]
    B.gtopk_dense_topk(dense, k, dev.g_idx, dev.g_val, B.alloc_workspace(m, k, 1))
    assert idx_np(dev.g_idx).tolist() == ex["alg2_g_idx"] and val_np(dev.g_val).tolist() == ex["alg2_g_val"]
    dev.set_res(np.array(ex["residual_after_select"], dtype=np.float32))
    dev.restore()
    assert dev.residual().tolist() == ex["alg2_residual"]


def _random_shape_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        P = int(rng.choice([1, 2, 4, 8, 16]))
        m = int(rng.choice([rng.integers(1, 40), rng.integers(40, 3000), rng.integers(3000, 120_000)]))
        k = int(rng.choice([1, m, max(1, m // 1000), rng.integers(1, m + 1)]))
        kind = str(rng.choice(["gauss", "ties", "special", "zeros_mostly"]))
        pad = int(rng.choice([0, 0, 1, 3, 5]))
        cases.append((P, m, k, kind, pad))
    return cases


@pytest.mark.parametrize("general", [False, True])
@pytest.mark.parametrize("P,m,k,kind,pad", _random_shape_cases(48, 20260427))
def test_step_random_shapes(P, m, k, kind, pad, general):
    """Seeded random problem shapes (tiny rows, k = m, k = 1, odd strides) and value kinds,
    two iterations each with the residual carried."""
    rng = np.random.default_rng(P * 1_000_003 + m * 31 + k)
    dev = Device(P, m, k, stride=m + pad if pad else None)
    res = np.zeros((P, m), dtype=np.float32)
    dev.set_res(res)
    for it in range(2):
        if kind == "gauss":
            g = rng.standard_normal((P, m)).astype(np.float32)
        elif kind == "ties":
            g = rng.integers(-3, 4, (P, m)).astype(np.float32) * np.float32(0.5)
        elif kind == "special":
            g = np.stack([W.special_values(m, seed=int(rng.integers(0, 10_000))) for _ in range(P)])
        else:
            g = np.where(rng.random((P, m)) < 0.02, rng.standard_normal((P, m)), 0.0).astype(np.float32)
        dev.set_grad(g)
        say(f"random shape P={P} m={m} k={k} kind={kind} pad={pad} it={it} general={general}")
        gi, gv = dev.step_carry() if general else dev.step()
        exp = orc.step(res, g, k)
        assert np.array_equal(idx_np(dev.loc_idx), exp["loc_idx"])
        assert bits_equal(val_np(dev.loc_val), exp["loc_val"])
        assert np.array_equal(gi, exp["g_idx"]) and bits_equal(gv, exp["g_val"])
        assert bits_equal(dev.residual(), exp["residual"])
        res = exp["residual"]


def _fill(kind, P, m, rng):
    """One batch of gradients of a value kind of the seeded sweeps below."""
    if kind == "gauss":
        return (rng.standard_normal((P, m)) * 1e-3).astype(np.float32)
    if kind == "ties":
        return rng.integers(-3, 4, (P, m)).astype(np.float32) * np.float32(0.5)
    if kind == "special":
        return np.stack([W.special_values(m, seed=int(rng.integers(0, 10_000))) for _ in range(P)])
    if kind == "sparse":
        return np.where(rng.random((P, m)) < 0.02, rng.standard_normal((P, m)), 0.0).astype(np.float32)
    g = (rng.standard_normal((P, m)) * 1e-3).astype(np.float32)
    if kind == "gaps":                 # stretches of zeros: chunks of the row without any candidate
        for w in range(P):
            a = int(rng.integers(0, m))
            g[w, a:min(m, a + int(rng.integers(1, max(2, m // 3))))] = 0.0
            if rng.random() < 0.5:
                g[w, :min(m, 40_000)] = 0.0
    elif kind == "plateau":            # a large share of the row at one magnitude: ties at the k-th key
        for w in range(P):
            n = int(m * rng.uniform(0.05, 0.6))
            at = rng.choice(m, n, replace=False)
            g[w, at] = np.where(rng.random(n) < 0.5, -1, 1).astype(np.float32) * np.float32(0.25)
    elif kind == "shared":             # the workers' large entries coincide: merges of overlapping sets
        base = (rng.standard_normal(m) * 1e-3).astype(np.float32)
        g = (base[None, :] * rng.uniform(0.5, 1.5, (P, 1)) + rng.standard_normal((P, m)) * 1e-5).astype(np.float32)
    return g


_SWEEP_KINDS = ["gauss", "ties", "special", "sparse", "gaps", "plateau", "shared"]


def _small_path_cases(n, seed):
    """Shapes inside the few-launch path's limits (P <= 64, k <= 512, P * k <= 4096, m < 2^20)."""
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        P = int(rng.choice([1, 2, 4, 8, 16, 32, 64]))
        kmax = min(512, 4096 // P)
        k = int(rng.choice([1, 2, kmax, int(rng.integers(1, kmax + 1)), int(rng.integers(1, kmax + 1))]))
        m = int(rng.choice([rng.integers(k, k + 50), rng.integers(k, 5000 + k), rng.integers(5000, 200_000),
                            rng.integers(200_000, 1_048_573)]))
        cases.append((P, max(m, k), k, str(rng.choice(_SWEEP_KINDS)), int(rng.choice([0, 0, 1, 2, 3, 7]))))
    return cases


def _long_run_cases(n, seed):
    """Densities at which the candidates are selected run by run where the pass left them."""
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        P = int(rng.choice([1, 2, 4, 8]))
        m = int(rng.choice([rng.integers(40_000, 200_000), rng.integers(200_000, 1_500_000)]))
        rho = float(rng.choice([0.006, 0.01, 0.03, 0.1, 0.25, 0.5, 0.9]))
        cases.append((P, m, min(m, max(513, int(m * rho))), str(rng.choice(_SWEEP_KINDS)), int(rng.choice([0, 0, 1, 3]))))
    return cases


def _check_two_iterations(P, m, k, kind, pad, label):
    rng = np.random.default_rng(P * 1_000_003 + m * 31 + k)
    dev = Device(P, m, k, stride=m + pad if pad else None)
    res = np.zeros((P, m), dtype=np.float32)
    dev.set_res(res)
    for it in range(2):
        g = _fill(kind, P, m, rng)
        dev.set_grad(g)
        say(f"{label} P={P} m={m} k={k} kind={kind} pad={pad} it={it}")
        gi, gv = dev.step()
        exp = orc.step(res, g, k)
        assert np.array_equal(idx_np(dev.loc_idx), exp["loc_idx"]), first_diff(idx_np(dev.loc_idx), exp["loc_idx"])
        assert bits_equal(val_np(dev.loc_val), exp["loc_val"])
        assert np.array_equal(gi, exp["g_idx"]), first_diff(gi, exp["g_idx"])
        assert bits_equal(gv, exp["g_val"])
        out = dev.residual()
        assert bits_equal(out, exp["residual"]), first_diff(out, exp["residual"])
        res = exp["residual"]


@pytest.mark.parametrize("P,m,k,kind,pad", _small_path_cases(60, 20261127))
def test_step_random_shapes_few_launch_path(P, m, k, kind, pad):
    """Seeded shapes and value kinds inside the limits of gtopk_step's few-launch path."""
    from paper_1901_04359_amd import binding as B
    assert B.gtopk_debug_plan(m, k, P)["small_path"] == 1
    _check_two_iterations(P, m, k, kind, pad, "few-launch sweep")


@pytest.mark.parametrize("P,m,k,kind,pad", _long_run_cases(30, 20261128))
def test_step_random_shapes_long_runs(P, m, k, kind, pad):
    """Seeded shapes and value kinds at the densities where the candidates are selected in place."""
    from paper_1901_04359_amd import binding as B
    plan = B.gtopk_debug_plan(m, k, P)
    assert plan["small_path"] == 0 and plan["run_groups"] == 1
    _check_two_iterations(P, m, k, kind, pad, "long-run sweep")


def _random_aggregation_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        P = int(rng.integers(1, 41))
        m = int(rng.choice([rng.integers(1, 60), rng.integers(60, 9000), rng.integers(9000, 200_000)]))
        k = int(rng.choice([1, m, max(1, m // 500), rng.integers(1, m + 1)]))
        k = min(k, 30_000)
        cases.append((P, m, k, float(rng.choice([0.0, 0.3, 0.9, 1.0])),
                      str(rng.choice(["gauss", "ties", "cancel"]))))
    return cases


@pytest.mark.parametrize("P,m,k,overlap,kind", _random_aggregation_cases(24, 20260428))
def test_aggregations_random_shapes(P, m, k, overlap, kind):
    """Algorithm 1's all-reduce for any worker count, then Algorithm 2's top-k of its result."""
    import torch
    from paper_1901_04359_amd import binding as B
    idx, val = W.ksets(P, k, m, seed=P * 7919 + k, overlap=overlap, value_kind=kind)
    say(f"random aggregation P={P} m={m} k={k} overlap={overlap} kind={kind}")
    dense = run_allreduce(idx, val, m)
    exp = orc.topk_allreduce(list(idx), list(val), m)
    got = dense.cpu().numpy()
    assert bits_equal(got, exp), first_diff(got, exp)
    g_idx = torch.zeros(k, dtype=torch.int32, device="cuda")
    g_val = torch.zeros(k, dtype=torch.float32, device="cuda")
    ws = B.alloc_workspace(m, k, 1)
    ws.fill_(0x5A)
    B.gtopk_dense_topk(dense, k, g_idx, g_val, ws)
    oi, ov = orc.dense_topk(exp, k)
    assert np.array_equal(idx_np(g_idx), oi) and bits_equal(val_np(g_val), ov)


def test_step_under_graph_capture():
    """gtopk_step allocates nothing, never synchronises and clears its workspace with a kernel
    of its own, so a caller may capture it in a HIP graph.  Three replays with eager work and
    synchronisations in between, each compared with the oracle (residual carried)."""
    import torch
    cfg = W.scaled(W.CONFIGS["C2"], 150_001, k=300, P=8, name="graph")
    P, m, k = cfg.P, cfg.m, cfg.k
    dev = Device(P, m, k)
    grads = [W.gradients(cfg, it) for it in range(3)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):            # warm-up outside capture, as torch asks
        dev.set_grad(grads[0])
        dev.step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    say("graph capture of gtopk_step")
    with torch.cuda.graph(graph):
        dev.B.gtopk_step(dev.grad, dev.res, k, dev.g_idx, dev.g_val, dev.loc_idx, dev.loc_val, dev.ws)
    res = np.zeros((P, m), dtype=np.float32)
    dev.set_res(res)
    for it in range(3):
        dev.set_grad(grads[it])
        scratch = torch.rand(1000, device="cuda").sum()      # eager work between the replays
        torch.cuda.synchronize()
        say(f"graph replay {it}")
        graph.replay()
        torch.cuda.synchronize()
        exp = orc.step(res, grads[it], k)
        assert np.array_equal(idx_np(dev.g_idx), exp["g_idx"]), it
        assert bits_equal(val_np(dev.g_val), exp["g_val"]), it
        assert np.array_equal(idx_np(dev.loc_idx), exp["loc_idx"]), it
        assert bits_equal(dev.residual(), exp["residual"]), it
        res = exp["residual"]
        assert float(scratch) > 0


def test_non_finite_inputs_keep_the_structure():
    """NaN / Inf are outside the method's domain (results unspecified), but every decision is
    taken on integer keys, so the outputs keep their structure: k ascending, distinct indices
    per worker, values copied from the accumulated row, and the global set drawn from the
    union of the local ones."""
    P, m, k = 4, 50_000, 100
    rng = np.random.default_rng(5)
    g = rng.standard_normal((P, m)).astype(np.float32)
    g[:, ::97] = np.inf
    g[:, 5::389] = -np.inf
    g[:, 11::1013] = np.nan
    dev = Device(P, m, k)
    dev.set_grad(g)
    say("non-finite inputs")
    gi, gv = dev.step()
    li = idx_np(dev.loc_idx)
    for w in range(P):
        assert (np.diff(li[w].astype(np.int64)) > 0).all() and li[w].max() < m
        # the selected entries are the non-finite ones: their keys are the largest
        assert (~np.isfinite(g[w][li[w]])).all()
    assert (np.diff(gi.astype(np.int64)) > 0).all()
    assert np.isin(gi, np.unique(li)).all()


@pytest.mark.parametrize("k", [300, 70_000, 600_000, 4_300_000])      # one size per union kernel
def test_merge_of_unsorted_sets_stays_in_bounds(k):
    """Unsorted or duplicate indices in caller-supplied sets give unspecified results, but the
    call must complete and leave neighbouring memory alone (guard words around the output)."""
    import torch
    from paper_1901_04359_amd import binding as B
    rng = np.random.default_rng(k)
    batch = 2
    mk = lambda: to_dev(rng.integers(0, 2 * k, (batch, k)).astype(np.uint32))
    a_idx, b_idx = mk(), mk()
    a_val = to_dev(rng.standard_normal((batch, k)).astype(np.float32))
    b_val = to_dev(rng.standard_normal((batch, k)).astype(np.float32))
    guard = 1024
    out_idx = torch.full((batch * k + 2 * guard,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    out_val = torch.full((batch * k + 2 * guard,), 7.0, dtype=torch.float32, device="cuda")
    ws = B.alloc_merge_workspace(k, batch)
    say(f"merge of unsorted sets k={k}")
    B.gtopk_merge(a_idx, a_val, b_idx, b_val, k, batch, k, out_idx[guard:guard + batch * k],
                  out_val[guard:guard + batch * k], k, ws)
    torch.cuda.synchronize()
    assert bool((out_idx[:guard] == 0x5A5A5A5A).all()) and bool((out_idx[-guard:] == 0x5A5A5A5A).all())
    assert bool((out_val[:guard] == 7.0).all()) and bool((out_val[-guard:] == 7.0).all())


def test_allreduce_of_unsorted_sets_stays_in_bounds():
    """The same for the all-reduce: unsorted, duplicate and out-of-range indices."""
    import torch
    from paper_1901_04359_amd import binding as B
    rng = np.random.default_rng(9)
    P, k, m = 5, 20_000, 100_000
    idx = to_dev(rng.integers(0, 2 * m, (P, k)).astype(np.uint32))
    val = to_dev(rng.standard_normal((P, k)).astype(np.float32))
    guard = 1024
    buf = torch.full((m + 2 * guard,), 7.0, dtype=torch.float32, device="cuda")
    ws = B.alloc_allreduce_workspace(m, P)
    say("all-reduce of unsorted sets")
    B.gtopk_topk_allreduce(idx, val, P, k, buf[guard:guard + m], ws)
    torch.cuda.synchronize()
    assert bool((buf[:guard] == 7.0).all()) and bool((buf[-guard:] == 7.0).all())
    assert bool(torch.isfinite(buf[guard:guard + m]).all())


def test_probe_stream_modes():
    """The bandwidth probe (instrumentation of the benchmark): every add form leaves b + a in b,
    one IEEE add per element, whatever its cache policy and block shape; the read-only form
    leaves both arrays alone and writes one finite float per 32768 elements."""
    import torch
    from paper_1901_04359_amd import binding as B
    n = 5 * 32768
    rng = np.random.default_rng(3)
    a = rng.standard_normal(n).astype(np.float32)
    b0 = rng.standard_normal(n).astype(np.float32)
    da = to_dev(a)
    for mode in (0, 2, 3, 4, 5, 6, 7):
        db = to_dev(b0)
        say(f"probe mode {mode}")
        B.gtopk_probe_stream(da, db, n, mode, None)
        torch.cuda.synchronize()
        assert bits_equal(val_np(db), b0 + a), f"mode {mode}: {first_diff(val_np(db), b0 + a)}"
        assert bits_equal(val_np(da), a)
    db = to_dev(b0)
    sink = torch.full((n // 32768,), float("nan"), dtype=torch.float32, device="cuda")
    B.gtopk_probe_stream(da, db, n, 1, sink)
    torch.cuda.synchronize()
    assert bits_equal(val_np(db), b0) and bits_equal(val_np(da), a)
    assert np.isfinite(val_np(sink)).all()
