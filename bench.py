#!/usr/bin/env python3
"""Benchmark of the gTop-k hot path on one MI355X.

A "step" is one pass of the whole hot path (gtopk_step: local select for all P
workers, log2 P merge rounds, division by P, residual restore) over one batch
of synthetic gradients that is already resident in HBM.  The workload is the
ResNet-50-sized configuration (m = 25,557,032 per worker, P = 32, k = 25,557).
Successive steps feed on different gradient batches and on the residual the
previous step left, as in training.

Prints ONE JSON line.  `value` = P*m / t_step (gradient elements per second).
`roofline` prices the dominant kernel (the streaming accumulate/filter pass)
against HBM: algorithmic bytes = 12 per gradient element (read gradient, read
residual, write residual), duration from HIP events recorded by the library
around that kernel in a second, equally long pass over the same steps (the event
records themselves cost about 30 us per step, so the pass that gives `value`
runs without them; `ms_per_step_with_stage_events` is the second pass).  `cpu_baseline` times the CPU oracle
on a bounded sample of the same workload (a few whole workers).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
N_STAGES = 6
STAGE_NAMES = ["sample", "accumulate_filter", "exact_select", "tree", "restore"]


def read_traffic_note(workload: str, what: str = "traffic_bytes_per_launch"):
    """HBM bytes per launch of the dominant kernel (or per step), from the committed
    rocprofv3 --pmc summary (a line `<what> <workload> <bytes>`), or None."""
    path = os.path.join(ROOT, "profiles", "k_accum_filter_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 3 and f[0] == what and f[1] == workload:
                return float(f[2])
    except OSError:
        pass
    return None


def cpu_baseline(cfg, n_workers: int, budget_s: float = 20.0):
    """The oracle as it stands on the first n_workers workers of the config (a power of
    two, so that the tree is a real one), its independent calls (workers in the selection
    and the restore, pairs of a tree round) spread over the host's cores with a thread
    pool; the same sample once more on one thread as a second, labelled figure.
    n_workers < 0: probe one worker's local selection first and take as many workers as
    fit in about `budget_s` seconds of CPU work for the two runs together."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import gtopk_oracle as orc
    from paper_1901_04359_amd import workloads as W
    cores = max(1, min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0)
                       or (os.cpu_count() or 1)))
    if n_workers < 0:
        g1 = W.gradient(cfg, 0, 0)
        t0 = time.perf_counter()
        orc.local_select(np.zeros_like(g1), g1, cfg.k)
        per_worker = max(time.perf_counter() - t0, 1e-3)
        n_workers = 2
        # one single-threaded run plus one threaded run of the same sample
        while (n_workers * 2 <= cfg.P and
               n_workers * 2 * per_worker * 1.3 * (1.0 + 2.0 / cores) <= budget_s):
            n_workers *= 2
    g = W.gradients(cfg, 0, workers=range(n_workers))
    r = np.zeros_like(g)
    threads = min(cores, n_workers)
    with ThreadPoolExecutor(max_workers=threads) as ex:
        t0 = time.perf_counter()
        orc.step(r, g, cfg.k, map_fn=lambda f, it: list(ex.map(f, it)))
        dt_pool = time.perf_counter() - t0
    t0 = time.perf_counter()
    orc.step(r, g, cfg.k)
    dt_one = time.perf_counter() - t0
    what = (f"oracle.step on {n_workers} of the {cfg.P} workers at full m={cfg.m}, k={cfg.k} "
            f"(select, {n_workers.bit_length() - 1}-round tree, restore), one iteration")
    return {
        "value": n_workers * cfg.m / dt_pool, "unit": "gradient elements/s", "cores": threads,
        "kind": "oracle",
        "sample": (f"{what}, {dt_pool:.1f} s with its independent calls on a pool of {threads} "
                   f"threads (numpy releases the GIL in its sorts); host reports "
                   f"{os.cpu_count()} cpus"),
        "single_thread": {"value": n_workers * cfg.m / dt_one, "cores": 1,
                          "sample": f"the same sample on one thread, {dt_one:.1f} s"},
    }


def hbm_ceiling(B, torch, a, b, reps: int = 20):
    """What the memory system gives to the streaming pass's access pattern, on the same two
    buffers the step streams (outside the timed region): the library's probe kernel in its
    add form (`b += a`: 8 bytes read, 4 written per element, exactly the pass's algorithmic
    traffic) and in its read-only form, and torch's own `b.add_(a)` as an independent
    reference.  HIP events on the current stream, `reps` launches each."""
    n = (a.numel() // 32768) * 32768
    av, bv = a.view(-1), b.view(-1)
    sink = torch.zeros(n // 32768, dtype=torch.float32, device="cuda")

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    t_add = timed(lambda: B.gtopk_probe_stream(av, bv, n, 0, None))
    t_read = timed(lambda: B.gtopk_probe_stream(av, bv, n, 1, sink))
    t_torch = timed(lambda: bv.add_(av))
    gbs = lambda nbytes, ms: round(nbytes / (ms * 1e-3) / 1e9, 1)
    # the add form with one of the pass's choices changed at a time (cache policy, block shape)
    variants = {"temporal_loads": 2, "temporal_stores": 3, "temporal_loads_and_stores": 4,
                "256_threads_x_32": 5, "1024_threads_x_8": 6, "8192_element_blocks": 7}
    sweep = {name: gbs(12.0 * n, timed(lambda md=md: B.gtopk_probe_stream(av, bv, n, md, None)))
             for name, md in variants.items()}
    return {
        "elements": n,
        "probe_add_GBs": gbs(12.0 * n, t_add), "probe_add_ms": round(t_add, 4),
        "probe_read_GBs": gbs(8.0 * n, t_read), "probe_read_ms": round(t_read, 4),
        "torch_add_GBs": gbs(12.0 * a.numel(), t_torch), "torch_add_ms": round(t_torch, 4),
        "probe_add_variants_GBs": sweep,
        "note": ("probe = k_probe_stream, the streaming pass's block shape and cache policy with "
                 "only the memory traffic left; add: 12 B per element, read: 8 B per element; "
                 "torch_add = torch's b.add_(a) on the same buffers; probe_add_variants = the add "
                 "form with one choice changed: ordinary instead of non-temporal loads / stores, "
                 "other block shapes (the pass: 512 threads x 16 accesses, 32768 elements per block)"),
    }


def time_aggregations(B, torch, cfg, grads, reps: int = 20):
    """The three ways of aggregating the P local k-sets that the paper compares, timed on the
    local sets of one step of this workload (HIP events, `reps` repetitions each):
    the gTop-k tree (Algorithm 3), Top-k S-SGD's TopKAllReduce (Algorithm 1: dense average),
    and the naive gTop-k (Algorithm 2: that average, then its top-k).  Also how many of the
    tree's k indices are in the naive version's exact global top-k."""
    P, m, k = cfg.P, cfg.m, cfg.k
    res = torch.zeros((P, m), dtype=torch.float32, device="cuda")
    loc_idx = torch.zeros((P, k), dtype=torch.int32, device="cuda")
    loc_val = torch.zeros((P, k), dtype=torch.float32, device="cuda")
    g_idx = torch.zeros(k, dtype=torch.int32, device="cuda")
    g_val = torch.zeros(k, dtype=torch.float32, device="cuda")
    n_idx = torch.zeros(k, dtype=torch.int32, device="cuda")
    n_val = torch.zeros(k, dtype=torch.float32, device="cuda")
    dense = torch.empty(m, dtype=torch.float32, device="cuda")
    ws = B.alloc_workspace(m, k, P)
    ws1 = B.alloc_workspace(m, k, 1)
    ws_ar = B.alloc_allreduce_workspace(m, P)
    B.gtopk_local_select(grads[0], res, k, loc_idx, loc_val, ws)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    t_tree = timed(lambda: B.gtopk_tree(loc_idx, loc_val, P, k, g_idx, g_val, ws))
    t_ar = timed(lambda: B.gtopk_topk_allreduce(loc_idx, loc_val, P, k, dense, ws_ar))
    t_top = timed(lambda: B.gtopk_dense_topk(dense, k, n_idx, n_val, ws1))
    shared = int(torch.isin(g_idx, n_idx).sum().item())
    ar_bytes = 4.0 * m + 8.0 * P * k
    return {
        "gtopk_tree_ms": round(t_tree, 4),
        "alg1_topk_allreduce_ms": round(t_ar, 4),
        "alg1_algorithmic_GBs": round(ar_bytes / (t_ar * 1e-3) / 1e9, 1),
        "alg2_dense_topk_ms": round(t_top, 4),
        "alg2_total_ms": round(t_ar + t_top, 4),
        "tree_indices_in_exact_global_topk": shared / k,
        "note": "alg1 bytes = 4*m (dense out) + 8*P*k (sets in); alg2 total = alg1 + its top-k",
    }


def time_three_calls(B, torch, cfg, grads, res, g_idx, g_val, ws, reps: int = 10):
    """gtopk_local_select, gtopk_tree and gtopk_residual_restore timed one by one (HIP events,
    `reps` repetitions each; the residual keeps evolving, as in training)."""
    P, k = cfg.P, cfg.k
    loc_idx = torch.zeros((P, k), dtype=torch.int32, device="cuda")
    loc_val = torch.zeros((P, k), dtype=torch.float32, device="cuda")

    def timed(fn):
        fn(0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            fn(i + 1)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    t_sel = timed(lambda i: B.gtopk_local_select(grads[i % len(grads)], res, k, loc_idx, loc_val, ws))
    t_tree = timed(lambda i: B.gtopk_tree(loc_idx, loc_val, P, k, g_idx, g_val, ws))
    t_res = timed(lambda i: B.gtopk_residual_restore(res, k, loc_idx, loc_val, g_idx))
    return {"gtopk_local_select_ms": round(t_sel, 4), "gtopk_tree_ms": round(t_tree, 4),
            "gtopk_residual_restore_ms": round(t_res, 4),
            "sum_ms": round(t_sel + t_tree + t_res, 4)}


def time_per_iteration(B, torch, W, cfg, reps: int = 20):
    """The config's own iterations (1 .. cfg.iters), each timed `reps` times from the residual the
    previous iteration left (restored from a saved copy outside the timed region): iteration 1
    starts from a zero residual, the later ones are the steady state."""
    P, m, k = cfg.P, cfg.m, cfg.k
    grads = [torch.from_numpy(W.gradients(cfg, it, threads=min(16, os.cpu_count() or 8))).cuda()
             for it in range(cfg.iters)]
    res = torch.zeros((P, m), dtype=torch.float32, device="cuda")
    saved = torch.zeros_like(res)
    g_idx = torch.zeros(k, dtype=torch.int32, device="cuda")
    g_val = torch.zeros(k, dtype=torch.float32, device="cuda")
    ws = B.alloc_workspace(m, k, P)
    out = {}
    for it in range(cfg.iters):
        saved.copy_(res)
        times = []
        for rep in range(reps + 2):
            res.copy_(saved)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            B.gtopk_step(grads[it], res, k, g_idx, g_val, None, None, ws)
            e1.record()
            torch.cuda.synchronize()
            if rep >= 2:
                times.append(e0.elapsed_time(e1))
        times.sort()
        out[str(it + 1)] = {"median_ms": round(times[len(times) // 2], 4), "min_ms": round(times[0], 4)}
        # res now holds the residual after iteration `it` (every repetition ends in the same state)
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C4a")
    ap.add_argument("--batches", type=int, default=2, help="distinct gradient batches staged in HBM")
    ap.add_argument("--k", type=int, default=0, help="override the workload's k (density studies)")
    ap.add_argument("--cpu-workers", type=int, default=-1,
                    help="workers in the oracle sample (0 = skip, -1 = as many as fit in ~15 s)")
    ap.add_argument("--per-iteration", action="store_true",
                    help="also time each of the config's iterations on its own, from the residual "
                         "its predecessor left (iteration 1: zero residual)")
    ap.add_argument("--three-calls", action="store_true",
                    help="also time gtopk_local_select, gtopk_tree and gtopk_residual_restore "
                         "one by one")
    ap.add_argument("--aggregations", action="store_true",
                    help="also time the paper's comparison aggregations (Algorithms 1 and 2) "
                         "against the tree on this workload's local sets")
    ap.add_argument("--degenerate-workers", type=int, default=0,
                    help="replace the gradient rows of this many workers by rows of equal "
                         "magnitudes, which overflow the candidate list and are selected from "
                         "the dense row (cost of the exact fallback)")
    ap.add_argument("--short-workers", type=int, default=0,
                    help="replace the gradient rows of this many workers by rows whose large "
                         "magnitudes sit only where the sampler looks, so that the speculative "
                         "threshold comes out too high, the pass keeps fewer than k candidates "
                         "and the worker is selected from its dense row (cost of a sampling miss)")
    ap.add_argument("--carry", action="store_true",
                    help="call gtopk_step_carry (speculative thresholds carried from step to step) "
                         "instead of gtopk_step (a fresh sample of every row on every step)")
    ap.add_argument("--no-ceiling", action="store_true",
                    help="skip the HBM-ceiling probe passes")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy a few times (reference "
                         "reading for the rocprofv3 FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all P workers are buffers on one device); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import torch
    from paper_1901_04359_amd import binding as B
    from paper_1901_04359_amd import workloads as W

    B.load()      # fails loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4,
                          "copies": 5}))
        return 0
    cfg = W.CONFIGS[args.workload]
    if args.k > 0:
        cfg = W.scaled(cfg, cfg.m, k=args.k, name=f"{cfg.name}/k={args.k}")
    P, m, k = cfg.P, cfg.m, cfg.k
    K, Wm = args.steps, args.warmup

    t_gen = time.perf_counter()
    grads = []
    for b in range(args.batches):
        host = W.gradients(cfg, b, threads=min(16, os.cpu_count() or 8))
        for w in range(min(args.degenerate_workers, P)):
            sign = np.random.default_rng(1000 * b + w).integers(0, 2, m).astype(np.float32) * 2 - 1
            host[(w * 7) % P] = sign * np.float32(0.125)
        if args.short_workers:
            plan = B.gtopk_debug_plan(m, k, P)
            t = np.arange(plan["n_tiles"], dtype=np.int64)[:, None] * plan["tile_stride"]
            pos = (t + np.arange(plan["tile_len"], dtype=np.int64)[None, :]).ravel()
            pos = pos[pos < m]
            n_big = min(pos.size, max(plan["target"] + plan["target"] // 3, min(k - 1, 2 * plan["target"])))
            for w in range(min(args.short_workers, P)):
                rng = np.random.default_rng(5000 * b + w)
                row = (rng.standard_normal(m) * 1e-3).astype(np.float32)
                at = rng.choice(pos, n_big, replace=False)
                row[at] = ((1.0 + rng.random(n_big)) * rng.choice([-1.0, 1.0], n_big)).astype(np.float32)
                host[(w * 7 + 3) % P] = row
        grads.append(torch.from_numpy(host).cuda())
        del host
    t_gen = time.perf_counter() - t_gen
    res = torch.zeros((P, m), dtype=torch.float32, device="cuda")
    g_idx = torch.zeros(k, dtype=torch.int32, device="cuda")
    g_val = torch.zeros(k, dtype=torch.float32, device="cuda")
    ws = B.alloc_workspace(m, k, P)

    # thresholds carried from step to step (zero: every worker starts from a sample)
    thr_state = None if not args.carry else torch.zeros((P, 4), dtype=torch.int32, device="cuda")

    def step(i: int) -> None:
        if thr_state is None:
            B.gtopk_step(grads[i % len(grads)], res, k, g_idx, g_val, None, None, ws)
        else:
            B.gtopk_step_carry(grads[i % len(grads)], res, k, g_idx, g_val, None, None, thr_state, ws)

    # stage events: created up front (a first record forces creation), recorded by the library
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(N_STAGES)] for _ in range(K)]
    for row in events:
        for e in row:
            e.record()
    for i in range(Wm):
        step(i)
    # the timed region: exactly K steps, nothing but the library's own launches in the stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step(Wm + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    modes_after_timed = None if thr_state is None else thr_state[:, 0].cpu().numpy().tolist()
    # the same K steps once more with the library recording its stage events (six event
    # records per step cost about 30 us, which is why they stay out of the region above):
    # stage times and the dominant kernel's duration come from here
    t2 = time.perf_counter()
    for i in range(K):
        B.gtopk_step_timed(grads[(Wm + K + i) % len(grads)], res, k, g_idx, g_val, None, None, ws,
                           [e.cuda_event for e in events[i]], thr_state)
    torch.cuda.synchronize()
    t3 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / K
    stage_ms = np.zeros(N_STAGES - 1)
    for row in events:
        for s in range(N_STAGES - 1):
            stage_ms[s] += row[s].elapsed_time(row[s + 1])
    stage_ms /= K
    step_gpu_ms = sorted(row[0].elapsed_time(row[N_STAGES - 1]) for row in events)
    value = P * m / (ms_per_step * 1e-3)

    kern_ms = float(stage_ms[1])
    alg_bytes = 12.0 * P * m
    achieved = alg_bytes / (kern_ms * 1e-3) / 1e9
    traffic = read_traffic_note(cfg.name)
    step_traffic = read_traffic_note(cfg.name, "traffic_bytes_per_step")
    label = {"C1": "tiny", "C2": "ResNet-20-sized", "C3": "VGG-16-sized", "C4a": "ResNet-50-sized",
             "C4b": "ResNet-50-sized", "C5": "AlexNet-sized"}.get(args.workload, "")
    out = {
        "metric": "gTop-k step throughput (P*m gradient elem/s) + achieved HBM GB/s vs peak",
        "value": value, "unit": "gradient elements/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": ms_per_step, "ms_per_step_with_stage_events": (t3 - t2) * 1e3 / K,
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {label}, m={m} fp32 per worker, P={P} workers "
                               f"on one GPU, k={k} (rho={cfg.rho:.4g}), {len(grads)} gradient "
                               f"batches cycled, residual carried across steps",
                   "m": m, "P": P, "k": k},
        "step_hbm": {"algorithmic_GBs": alg_bytes / (ms_per_step * 1e-3) / 1e9,
                     "frac_of_peak": alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "counter_GBs": (step_traffic / (ms_per_step * 1e-3) / 1e9
                                     if step_traffic else None)},
        "stages_ms": {n: round(float(v), 4) for n, v in zip(STAGE_NAMES, stage_ms)},
        "step_gpu_ms": {"median": round(step_gpu_ms[len(step_gpu_ms) // 2], 4),
                        "min": round(step_gpu_ms[0], 4), "max": round(step_gpu_ms[-1], 4),
                        "note": "per step of the second pass, first to last HIP event of the step"},
        "roofline": {"kernel": "k_accum_filter", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic,
                     "traffic_source": ("profiles/k_accum_filter_traffic.txt: rocprofv3 --pmc FETCH_SIZE / "
                                        "WRITE_SIZE per dispatch, scaled by a 1 GiB copy's readings; a "
                                        "committed summary, not measured in this run"
                                        if traffic else None),
                     "launch_ms": kern_ms,
                     "measured": "HIP events around the kernel in a second pass over the same K steps",
                     "algorithmic_bytes_per_launch": alg_bytes},
        "input_generation_s": round(t_gen, 1),
        "entry_point": "gtopk_step" if thr_state is None else "gtopk_step_carry",
    }
    if thr_state is None and B.gtopk_debug_plan(m, k, P)["small_path"]:
        out["stages_note"] = ("this problem is small enough for gtopk_step's few-launch path, which `value` "
                              "and ms_per_step time; the second pass (gtopk_step_timed) runs the general "
                              "kernels, so stages_ms and roofline describe those")
    if thr_state is not None:
        out["carried_thresholds"] = {
            "workers_not_sampling_after_timed_steps": sum(1 for md in modes_after_timed if md == 2),
            "workers": P,
            "note": ("gtopk_step_carry: same results as gtopk_step; a worker whose k-th magnitude "
                     "moves predictably filters with a threshold extrapolated from its previous "
                     "steps instead of sampling its row")}
    if args.degenerate_workers:
        counts, cap = B.gtopk_debug_candidate_counts(ws, m, k, P)
        out["degenerate_workers"] = {
            "requested": args.degenerate_workers,
            "served_from_dense_row_in_last_step": sum(1 for c in counts if c < k or c > cap)}
    if args.short_workers:
        counts, cap = B.gtopk_debug_candidate_counts(ws, m, k, P)
        out["short_workers"] = {
            "requested": args.short_workers,
            "with_fewer_than_k_candidates_in_last_step": sum(1 for c in counts if c < k)}
    if not args.no_ceiling:
        out["hbm_ceiling"] = hbm_ceiling(B, torch, grads[0], res)
        res.zero_()
    if args.three_calls:
        out["three_calls"] = time_three_calls(B, torch, cfg, grads, res, g_idx, g_val, ws)
    if args.aggregations:
        del res, ws
        out["aggregations"] = time_aggregations(B, torch, cfg, grads)
        res = ws = None
    if args.per_iteration:
        del res, ws, grads
        out["per_iteration"] = time_per_iteration(B, torch, W, cfg)
    if args.cpu_workers != 0:
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_workers)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
