"""Host-side check of the sampler's plan (no GPU): over random layer structures of the kind
the workloads are drawn from, the speculative threshold that the plan's sample would give
keeps at least k and at most `capacity` entries of the row - the condition under which a
worker is served from its candidate list and not from its dense row.

The plan (tile positions, target rank, list capacity) comes from the library through
gtopk_debug_plan; the estimate is modelled here with numpy: the threshold is the plan's
target-th largest magnitude among the sampled elements, rounded down to the edge of a
histogram bucket (the sampler's buckets are at most 1/64 of the magnitude wide).  A miss
would cost time only (the select is exact whatever it filters with), so this is a check of
the margin, not of correctness."""
import numpy as np
import pytest

from paper_1901_04359_amd import binding as B


def _row(rng, m, nseg):
    """Gaussian row in `nseg` contiguous segments: lengths from weights exp(U(0, ln 1000)),
    standard deviations log-uniform in [1e-5, 1e-2] (the recipe of the large configurations)."""
    w = np.exp(rng.uniform(0.0, np.log(1000.0), nseg))
    lens = np.maximum(1, (w / w.sum() * m).astype(np.int64))
    lens[-1] = m - lens[:-1].sum()
    assert lens[-1] > 0
    sig = np.exp(rng.uniform(np.log(1e-5), np.log(1e-2), nseg)).astype(np.float32)
    x = rng.standard_normal(m, dtype=np.float32)
    x *= np.repeat(sig, lens)
    return x


@pytest.mark.parametrize("nseg", [8, 54, 400])
@pytest.mark.parametrize("m,k", [(2_555_703, 2_556), (3_000_017, 30_000)])
def test_sample_plan_keeps_between_k_and_capacity(m, k, nseg):
    try:
        plan = B.gtopk_debug_plan(m, k, 32)
    except OSError as e:          # library not built
        pytest.skip(str(e))
    t = np.arange(plan["n_tiles"], dtype=np.int64)[:, None] * plan["tile_stride"]
    pos = (t + np.arange(plan["tile_len"], dtype=np.int64)[None, :]).ravel()
    pos = pos[pos < m]
    assert pos.size < m and plan["target"] <= pos.size
    ratios = []
    for trial in range(6):
        rng = np.random.default_rng(100 * nseg + trial)
        mag = np.abs(_row(rng, m, nseg))
        thr = np.sort(mag[pos])[::-1][plan["target"] - 1]
        kept = int((mag >= thr).sum())                               # with the exact sample key
        kept_lo = int((mag >= thr * np.float32(1.0 - 1.0 / 64)).sum())   # with a bucket edge below it
        assert kept >= k, f"trial {trial}: the threshold keeps {kept} < k = {k}"
        assert kept_lo <= plan["capacity"], f"trial {trial}: {kept_lo} > capacity {plan['capacity']}"
        ratios.append(kept_lo / k)
    assert max(ratios) < 2.5, ratios      # the margin is a fraction of k, not a multiple
