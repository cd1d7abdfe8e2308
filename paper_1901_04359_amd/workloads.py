"""Seeded synthetic inputs for the gTop-k hot path.

This module only *draws numbers*: gradient vectors shaped like the paper's
models (parameter counts of Table III's networks, a layer-wise scale
structure) and sparse (index, value) k-sets.  It holds none of the method's
arithmetic (no accumulate, no selection, no merge) and is the one module that
both the CPU oracle's tests and the HIP path's tests/bench may import, so
that both sides read identical bits.

The vectors stand in for real gradients of VGG-16 / ResNet-20 (Cifar-10) and
AlexNet / ResNet-50 (ImageNet); nothing from those datasets is reproduced.

Randomness: numpy's counter-based Philox generator, keyed by
(BASE_SEED, config, stream, iteration, worker).  Every (config, iteration,
worker) vector can be generated independently and in any order.
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 190104359

# stream ids (second key word) so that structure and values never share draws
_STREAM_STRUCTURE = 1
_STREAM_GRADIENT = 2
_STREAM_KSET = 3
_STREAM_SHARED = 4


@dataclasses.dataclass(frozen=True)
class Config:
    """One synthetic workload: m gradients per worker, P workers, k selected."""

    name: str
    cid: int            # numeric id mixed into the RNG key
    m: int
    P: int
    k: int
    iters: int
    kind: str           # "laplace" | "gauss" | "gauss_heavy" | "alexnet"
    n_segments: int = 1
    sigma_lo: float = 1e-3
    sigma_hi: float = 1e-3

    @property
    def rho(self) -> float:
        return self.k / self.m


CONFIGS: Dict[str, Config] = {
    "C1": Config("C1", 1, 65_536, 4, 66, 3, "laplace", 1, 1e-3, 1e-3),
    "C2": Config("C2", 2, 269_722, 8, 270, 5, "gauss", 22, 1e-4, 1e-2),
    "C3": Config("C3", 3, 14_728_266, 16, 14_728, 5, "gauss_heavy", 16, 1e-5, 1e-2),
    "C4a": Config("C4a", 4, 25_557_032, 32, 25_557, 5, "gauss", 54, 1e-5, 1e-2),
    "C4b": Config("C4b", 4, 25_557_032, 32, 255_570, 5, "gauss", 54, 1e-5, 1e-2),
    "C5": Config("C5", 5, 61_100_840, 32, 61_101, 5, "alexnet", 8, 1e-4, 1e-2),
}


def _rng(cid: int, stream: int, a: int = 0, b: int = 0) -> np.random.Generator:
    # Philox takes a 2x64-bit key; fold the five words into it reproducibly.
    k0 = (BASE_SEED << 20) ^ (cid << 8) ^ stream
    k1 = (a << 32) ^ b
    return np.random.Generator(np.random.Philox(key=[k0 & (2**64 - 1), k1 & (2**64 - 1)]))


def segment_layout(cfg: Config) -> Tuple[np.ndarray, np.ndarray]:
    """Segment lengths (int64, sum == m) and per-segment scale sigma_l (float32).

    Shared by all workers and iterations of a config (every worker trains the
    same model).  Lengths: weights exp(U(0, ln 1000)) normalised to m, the last
    segment takes the remainder.  Scales: log-uniform in [sigma_lo, sigma_hi].
    """
    m = cfg.m
    if cfg.kind == "laplace" or cfg.n_segments == 1:
        return np.array([m], dtype=np.int64), np.array([cfg.sigma_lo], dtype=np.float32)
    if cfg.kind == "alexnet":
        # five leading (convolution-like) segments share 4 % of m equally, sigma 1e-2;
        # three trailing fully-connected segments share the rest in the ratio of a
        # 9216x4096 : 4096x4096 : 4096x1000 stack, sigma 1e-4.
        lead_total = int(round(0.04 * m))
        lead = [lead_total // 5] * 5
        fc_w = np.array([9216 * 4096, 4096 * 4096, 4096 * 1000], dtype=np.float64)
        rest = m - sum(lead)
        fc = [int(rest * fc_w[0] / fc_w.sum()), int(rest * fc_w[1] / fc_w.sum())]
        fc.append(rest - sum(fc))
        lengths = np.array(lead + fc, dtype=np.int64)
        sig = np.array([cfg.sigma_hi] * 5 + [cfg.sigma_lo] * 3, dtype=np.float32)
        assert lengths.sum() == m and (lengths > 0).all()
        return lengths, sig
    r = _rng(cfg.cid, _STREAM_STRUCTURE)
    w = np.exp(r.uniform(0.0, math.log(1000.0), cfg.n_segments))
    lengths = np.floor(w / w.sum() * m).astype(np.int64)
    lengths = np.maximum(lengths, 1)
    lengths[-1] = m - lengths[:-1].sum()
    assert lengths[-1] > 0 and lengths.sum() == m
    sig = np.exp(r.uniform(math.log(cfg.sigma_lo), math.log(cfg.sigma_hi), cfg.n_segments))
    return lengths, sig.astype(np.float32)


_scale_cache: Dict[str, np.ndarray] = {}


def _scale_vector(cfg: Config) -> np.ndarray:
    key = f"{cfg.cid}:{cfg.m}"
    if key not in _scale_cache:
        lengths, sig = segment_layout(cfg)
        _scale_cache.clear()  # one big vector at a time is plenty
        _scale_cache[key] = np.repeat(sig, lengths).astype(np.float32)
    return _scale_cache[key]


def _laplace_unit(r: np.random.Generator, n: int) -> np.ndarray:
    """Laplace(0, 1) by inverse CDF from float32 uniforms."""
    u = r.random(n, dtype=np.float32) - np.float32(0.5)
    mag = -np.log1p(-np.minimum(np.float32(2.0) * np.abs(u), np.float32(1.0 - 2.0**-24)))
    return (np.sign(u) * mag).astype(np.float32)


def gradient(cfg: Config, iteration: int, worker: int) -> np.ndarray:
    """Fresh gradient vector (float32, length m) of `worker` at `iteration` (0-based)."""
    r = _rng(cfg.cid, _STREAM_GRADIENT, iteration, worker)
    m = cfg.m
    if cfg.kind == "laplace":
        return _laplace_unit(r, m) * np.float32(cfg.sigma_lo)
    scale = _scale_vector(cfg)
    g = r.standard_normal(m, dtype=np.float32)
    g *= scale
    if cfg.kind == "gauss_heavy":
        # 5 % of the entries come from a Laplace with ten times the segment's scale
        heavy = r.random(m, dtype=np.float32) < np.float32(0.05)
        lap = _laplace_unit(r, m)
        np.copyto(g, lap * (scale * np.float32(10.0)), where=heavy)
    elif cfg.kind == "alexnet":
        # 0.1 % of the values get their low 20 mantissa bits cleared: 8 magnitudes
        # per binade, so equal magnitudes occur at every scale (tie stress)
        q = r.random(m, dtype=np.float32) < np.float32(0.001)
        bits = g.view(np.uint32)
        np.copyto(bits, bits & np.uint32(0xFFF00000), where=q)
    return g


def gradients(cfg: Config, iteration: int, workers: Optional[Sequence[int]] = None,
              threads: int = 8, out: Optional[np.ndarray] = None) -> np.ndarray:
    """[len(workers)][m] float32 gradients of one iteration, generated in parallel."""
    if workers is None:
        workers = range(cfg.P)
    workers = list(workers)
    if out is None:
        out = np.empty((len(workers), cfg.m), dtype=np.float32)
    _scale_vector(cfg)  # build once, outside the pool

    def fill(j: int) -> None:
        out[j] = gradient(cfg, iteration, workers[j])

    if threads <= 1 or len(workers) == 1:
        for j in range(len(workers)):
            fill(j)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(len(workers))))
    return out


def scaled(cfg: Config, m: int, k: Optional[int] = None, P: Optional[int] = None,
           name: Optional[str] = None) -> Config:
    """Same recipe as `cfg` at another size (parity tests at oracle-friendly sizes)."""
    if k is None:
        k = max(1, int(round(cfg.rho * m)))
    return dataclasses.replace(cfg, m=m, k=k, P=cfg.P if P is None else P,
                               name=name or f"{cfg.name}@{m}")


# ----------------------------------------------------------------------------
# test-only generators (not configs)
# ----------------------------------------------------------------------------

def correlated_gradients(m: int, P: int, iteration: int, sigma: float = 1e-3,
                         seed: int = 7) -> np.ndarray:
    """Workers share a common component so merges meet matching indices often:
    g_w = sigma * (sqrt(1/2) z_shared + sqrt(1/2) z_w)."""
    shared = _rng(100 + seed, _STREAM_SHARED, iteration, 0).standard_normal(m, dtype=np.float32)
    out = np.empty((P, m), dtype=np.float32)
    c = np.float32(math.sqrt(0.5) * sigma)
    for w in range(P):
        own = _rng(100 + seed, _STREAM_GRADIENT, iteration, w).standard_normal(m, dtype=np.float32)
        out[w] = c * shared + c * own
    return out


def ksets(n_sets: int, k: int, m: int, seed: int = 0, overlap: float = 0.3,
          value_kind: str = "gauss") -> Tuple[np.ndarray, np.ndarray]:
    """`n_sets` sparse k-sets over [0, m): indices ascending and distinct (uint32
    [n_sets][k]), values float32.  A fraction `overlap` of each set's indices is
    drawn from a pool common to all sets, so that pairs of sets share indices.
    value_kind: "gauss" | "ties" (few distinct magnitudes, both signs) |
    "cancel" (shared indices carry opposite values in odd/even sets)."""
    assert 1 <= k <= m
    r0 = _rng(200 + seed, _STREAM_KSET, k, m & 0xFFFFFFFF)
    n_pool = min(m, max(1, int(round(overlap * k))))
    pool = np.sort(r0.choice(m, size=n_pool, replace=False)) if n_pool > 0 else np.empty(0, np.int64)
    idx = np.empty((n_sets, k), dtype=np.uint32)
    val = np.empty((n_sets, k), dtype=np.float32)
    for s in range(n_sets):
        r = _rng(200 + seed, _STREAM_KSET, s + 1, k)
        if k == m:
            chosen = np.arange(m, dtype=np.int64)
        else:
            n_sh = min(n_pool, int(round(overlap * k)))
            own_needed = k - n_sh
            # draw distinct indices outside the pool
            cand = r.choice(m, size=min(m, own_needed + n_pool + 16), replace=False)
            cand = cand[~np.isin(cand, pool)][:own_needed]
            if cand.size < own_needed:  # tiny m: fall back to any distinct completion
                rest = np.setdiff1d(np.arange(m), np.concatenate([pool[:n_sh], cand]))
                cand = np.concatenate([cand, r.permutation(rest)[: own_needed - cand.size]])
            chosen = np.concatenate([pool[:n_sh], cand])
        chosen = np.sort(chosen)
        assert chosen.size == k and (np.diff(chosen) > 0).all()
        idx[s] = chosen.astype(np.uint32)
        if value_kind == "gauss":
            v = r.standard_normal(k, dtype=np.float32) * np.float32(1e-3)
        elif value_kind == "ties":
            mags = np.array([1.0, 0.5, 0.25, 0.0], dtype=np.float32)
            v = mags[r.integers(0, 4, k)] * np.where(r.random(k) < 0.5, -1, 1).astype(np.float32)
        elif value_kind == "cancel":
            v = r.standard_normal(k, dtype=np.float32) * np.float32(1e-3)
            in_pool = np.isin(chosen, pool)
            base = ((chosen % 97).astype(np.float32) + np.float32(1.0)) * np.float32(1e-3)
            v = np.where(in_pool, base * np.float32(1.0 if s % 2 == 0 else -1.0), v).astype(np.float32)
        else:
            raise ValueError(value_kind)
        val[s] = v
    return idx, val


def special_values(m: int, seed: int = 0) -> np.ndarray:
    """A vector mixing denormals, +-0, repeated magnitudes and ordinary values."""
    r = _rng(300 + seed, _STREAM_GRADIENT, m & 0xFFFFFFFF, 0)
    g = r.standard_normal(m, dtype=np.float32) * np.float32(1e-3)
    kind = r.integers(0, 8, m)
    bits = g.view(np.uint32)
    # denormals: clear the exponent field
    np.copyto(bits, bits & np.uint32(0x807FFFFF), where=(kind == 0))
    g[kind == 1] = np.float32(0.0)
    g[kind == 2] = np.float32(-0.0)
    np.copyto(bits, bits & np.uint32(0xFFF00000), where=(kind == 3))
    return g
