"""GPU parity on the dense-row fallback of the local selection (Algorithm 4 lines 5-8).

The speculative threshold only sizes the work: a worker whose streaming pass kept fewer
than k candidates, or more than its list holds, is selected from its dense row.  These
tests force both outcomes, on rows far longer than the sampler's whole-row limit, at the
two ends of the density range where the pass histograms its own candidates (the fallback
then builds a histogram of its own) and in between, with fallback and ordinary workers
side by side in one launch.  Every output is compared bit for bit with the oracle, and
the candidate counts the pass left behind tell which path served each worker.

The rows are built from the layout that gtopk_debug_plan reports (tile positions of the
sampler, list capacity); none of the library's planning code is repeated here."""
import numpy as np
import pytest

from oracle import gtopk_oracle as orc
from paper_1901_04359_amd import workloads as W
from tests.gpu_harness import Device, bits_equal, first_diff, say, idx_np, val_np

pytestmark = pytest.mark.gpu

# expected path of a row kind: "cand" (served from the candidate list), "over" (more
# candidates than the list holds), "under" (fewer than k candidates)
KINDS = ["gauss", "all_equal", "under", "few_levels", "all_zero", "one_spike", "plateau", "gap"]


def sampled_positions(plan, m):
    t = np.arange(plan["n_tiles"], dtype=np.int64)[:, None] * plan["tile_stride"]
    pos = (t + np.arange(plan["tile_len"], dtype=np.int64)[None, :]).ravel()
    return pos[pos < m]


def make_row(kind, m, k, plan, rng, base):
    """(row, expected path).  `base` is an ordinary gradient row of the C4a recipe."""
    if kind == "gauss":
        return base, "cand"
    if kind == "all_equal":            # every magnitude ties: the lowest k indices win
        return (np.where(rng.random(m) < 0.5, -1, 1).astype(np.float32) * np.float32(0.125)), "over"
    if kind == "all_zero":
        g = np.zeros(m, dtype=np.float32)
        g[::3] = -0.0
        return g, "over"
    if kind == "one_spike":
        g = np.zeros(m, dtype=np.float32)
        g[m // 3] = 7.0
        return g, "over"
    if kind == "few_levels":
        # one magnitude held by two thirds of the row: more than any list holds, and the
        # k-th key ties with hundreds of thousands of others
        return rng.integers(-1, 2, m).astype(np.float32) * np.float32(0.5), "over"
    if kind == "gap":
        # an ordinary row whose first 70,000 elements and a stretch in the middle are zero: the
        # chunks there leave no candidates at all
        g = base.copy()
        g[:70_000] = 0.0
        g[m // 2: m // 2 + 40_000] = 0.0
        return g, "cand"
    if kind == "plateau":
        # three tenths of the row share one magnitude far above the rest: where the list holds
        # them they are candidates, the k-th key ties with all of them (more than the select's
        # list of in-bin keys holds), and the ties run across the whole row
        n_plat = (3 * m) // 10
        g = (rng.standard_normal(m) * 1e-3).astype(np.float32)
        at = rng.choice(m, n_plat, replace=False)
        g[at] = np.where(rng.random(n_plat) < 0.5, -1, 1).astype(np.float32) * np.float32(0.5)
        return g, ("cand" if k <= n_plat <= plan["capacity"] else "over")
    if kind == "under":
        # large magnitudes ONLY where the sampler looks: the sample sees the same number of
        # them as the whole row holds and puts the threshold among them, so the pass keeps
        # fewer than k entries
        pos = sampled_positions(plan, m)
        target = plan["target"]
        n_big = min(pos.size, max(target + target // 3, min(k - 1, 2 * target)))
        assert target < n_big and pos.size < m
        g = (rng.standard_normal(m) * 1e-3).astype(np.float32)
        at = pos if n_big >= pos.size else rng.choice(pos, n_big, replace=False)
        mag = (1.0 + rng.random(at.size)).astype(np.float32)          # distinct-ish keys in [1, 2)
        g[at] = mag * np.where(rng.random(at.size) < 0.5, -1, 1).astype(np.float32)
        return g, "under"
    raise ValueError(kind)


def build_case(m, k, P, seed):
    from paper_1901_04359_amd import binding as B
    plan = B.gtopk_debug_plan(m, k, P)
    cfg = W.scaled(W.CONFIGS["C4a"], m, k=k, P=P, name=f"fallback m={m} k={k}")
    rng = np.random.default_rng(seed)
    base = W.gradients(cfg, 0)
    rows, paths = [], []
    for w in range(P):
        row, path = make_row(KINDS[w % len(KINDS)], m, k, plan, rng, base[w])
        rows.append(row)
        paths.append(path)
    return cfg, plan, np.stack(rows), paths


def check_paths(counts, cap, k, paths, label):
    for w, (c, path) in enumerate(zip(counts, paths)):
        got = "under" if c < k else ("over" if c > cap else "cand")
        assert got == path, f"{label}: worker {w} count {c} (k={k}, cap={cap}) took '{got}', wanted '{path}'"


# (m, k, P, histogram regime of the streaming pass); the first case copies its candidates into
# index order, the others select them run by run where the pass left them
CASES = [
    (1_000_003, 1000, 8, 1),          # rho = 0.001: the pass histograms (few candidates per block)
    (1_000_003, 125_000, 8, 1),       # rho = 1/8: the pass histograms (very many per block)
    (1_000_003, 15_000, 8, 0),        # rho = 0.015: the select's histogram kernel does
    (700_001, 700, 4, 1),             # a second shape, P = 4
    (3_000_017, 30_000, 32, 0),       # rho = 0.01, 32 workers: one group per run of the pass
]


@pytest.mark.parametrize("m,k,P,pass_hist", CASES)
def test_fallback_step_mixed_workers(m, k, P, pass_hist):
    from paper_1901_04359_amd import binding as B
    cfg, plan, g0, paths = build_case(m, k, P, seed=m + k)
    if not plan["small_path"]:
        assert plan["pass_histogram"] == pass_hist, plan
        assert plan["run_groups"] == (1 if k * 1000 >= 6 * m else 0), plan
    assert plan["n_tiles"] * plan["tile_len"] < m, "the sampler must not see the whole row"
    dev = Device(P, m, k)
    res = np.zeros((P, m), dtype=np.float32)
    dev.set_res(res)
    rng = np.random.default_rng(7)
    for it in range(2):
        # second iteration: fresh ordinary gradients on top of the residual the first left
        g = g0 if it == 0 else W.gradients(cfg, 1)
        if it == 1:
            for w, p in enumerate(paths):
                if p == "over":                      # keep the degenerate rows degenerate
                    g[w] = 0.0
                    res[w] = g0[w] * np.float32(2.0)
            dev.set_res(res)
        dev.set_grad(g)
        say(f"fallback step m={m} k={k} P={P} it={it}")
        gi, gv = dev.step()
        counts, cap = B.gtopk_debug_candidate_counts(dev.ws, m, k, P)
        assert cap == plan["capacity"]
        exp = orc.step(res, g, k)
        li, lv = idx_np(dev.loc_idx), val_np(dev.loc_val)
        for w in range(P):
            assert np.array_equal(li[w], exp["loc_idx"][w]), \
                f"it={it} w={w} ({paths[w]}) loc_idx {first_diff(li[w], exp['loc_idx'][w])}"
            assert bits_equal(lv[w], exp["loc_val"][w]), \
                f"it={it} w={w} ({paths[w]}) loc_val {first_diff(lv[w], exp['loc_val'][w])}"
        assert np.array_equal(gi, exp["g_idx"]), f"it={it} g_idx {first_diff(gi, exp['g_idx'])}"
        assert bits_equal(gv, exp["g_val"]), f"it={it} g_val {first_diff(gv, exp['g_val'])}"
        out = dev.residual()
        for w in range(P):
            assert bits_equal(out[w], exp["residual"][w]), \
                f"it={it} w={w} ({paths[w]}) residual {first_diff(out[w], exp['residual'][w])}"
        if it == 0:
            check_paths(counts, cap, k, paths, f"step m={m} k={k}")
        else:
            # the degenerate rows still overflow; every path that ran was checked above
            for w, p in enumerate(paths):
                if p == "over":
                    assert counts[w] > cap, (w, counts[w], cap)
        res = exp["residual"]


@pytest.mark.parametrize("m,k,P,pass_hist", CASES[:3])
def test_fallback_local_select_mixed_workers(m, k, P, pass_hist):
    """The same rows through the stand-alone gtopk_local_select (which also zeroes the
    selected entries of a dense row after the select has read it)."""
    from paper_1901_04359_amd import binding as B
    cfg, plan, g, paths = build_case(m, k, P, seed=m + k)
    dev = Device(P, m, k)
    res = np.zeros((P, m), dtype=np.float32)
    dev.set_res(res)
    dev.set_grad(g)
    say(f"fallback local_select m={m} k={k} P={P}")
    gi, gv = dev.local_select()
    counts, cap = B.gtopk_debug_candidate_counts(dev.ws, m, k, P)
    check_paths(counts, cap, k, paths, f"local_select m={m} k={k}")
    out = dev.residual()
    for w in range(P):
        oi, ov, ores = orc.local_select(res[w], g[w], k)
        assert np.array_equal(gi[w], oi), f"w={w} ({paths[w]}) idx {first_diff(gi[w], oi)}"
        assert bits_equal(gv[w], ov), f"w={w} ({paths[w]}) val {first_diff(gv[w], ov)}"
        assert bits_equal(out[w], ores), f"w={w} ({paths[w]}) residual {first_diff(out[w], ores)}"


def test_fallback_every_worker_under_count():
    """All workers miss at once (no ordinary worker in the launch), unaligned rows."""
    from paper_1901_04359_amd import binding as B
    P, m, k = 4, 600_011, 600
    plan = B.gtopk_debug_plan(m, k, P)
    rng = np.random.default_rng(11)
    g = np.stack([make_row("under", m, k, plan, rng, None)[0] for _ in range(P)])
    dev = Device(P, m, k, stride=m + 3)
    res = np.zeros((P, m), dtype=np.float32)
    dev.set_grad(g)
    say(f"fallback all-under m={m} k={k} P={P}")
    gi, gv = dev.step()
    counts, cap = B.gtopk_debug_candidate_counts(dev.ws, m, k, P)
    assert all(c < k for c in counts), (counts, k)
    exp = orc.step(res, g, k)
    assert np.array_equal(idx_np(dev.loc_idx), exp["loc_idx"])
    assert bits_equal(val_np(dev.loc_val), exp["loc_val"])
    assert np.array_equal(gi, exp["g_idx"]) and bits_equal(gv, exp["g_val"])
    assert bits_equal(dev.residual(), exp["residual"])
