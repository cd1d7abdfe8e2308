"""CPU oracle for the gTop-k S-SGD data-parallel hot path (numpy, fp32).

THIS IS TEST INFRASTRUCTURE.  Only tests, the smoke check and the benchmark's
`cpu_baseline` leg may import it.  It shares no code with the HIP library and
imports nothing from the product package; inputs arrive as numpy arrays.

Every function is the plain definition of one step of the method (a full sort
wherever something is selected, no blocking, no approximation), and the steps
are composed in the order the paper gives them, so that each can be checked
against its passage by eye:

  * Algorithm 4 (the S-SGD iteration built on gTopKAllReduce), its local part:
    accumulate, threshold, mask, extract, keep residual  -> `local_select`
  * Definition 1 (the Top-k operation between two sparse vectors) -> `merge`
  * Algorithm 3 (gTopKAllReduce), the rounds of the binary tree  -> `tree`
  * Eq. 3 (S-SGD averages over the P workers)                  -> the /P in `tree`
  * Algorithm 3's broadcast and gMask, Algorithm 4's extra-residual
    step                                                        -> `residual_restore`
  * Algorithm 4's model update and the dense gMask              -> `apply_update`, `dense_mask`
  * The two aggregations the paper compares against, as comparison workloads:
    Algorithm 1, procedure TopKAllReduce (gather, scatter-add, average)
                                                                 -> `topk_allreduce`
    Algorithm 2 (naive gTop-k): the top-k of that dense average
                                                                 -> `dense_topk`

Precision: the paper trains in 32-bit floating point (note under Table III), so
every add here is ONE IEEE-754 binary32 round-to-nearest add, in a fixed order;
magnitudes are compared on the integer bit pattern, so no floating-point
comparison decides anything.

Readings taken where the paper is silent or inconsistent:

  R1  Algorithm 4's threshold and mask steps compare `|G| > thr` with thr the
      k-th largest magnitude, which taken literally selects k-1 entries, while
      the listing's own remark gives the mask k of them.  The remark wins: exactly k
      entries are selected, the first k under the total order (|v| descending,
      index ascending).
  R2  |v| is compared as the unsigned integer `bits(v) & 0x7fffffff`
      (monotone in |v| for finite values; +0 and -0 are equal).
  R4  A merge selects among the UNION OF INDICES of its two operands, whatever
      the summed values are (a sum may cancel to 0 and is still a candidate),
      so every merge output has exactly k entries.
  R5  Ranks are 0-based; in round j (j = 0 .. log2 P - 1) worker i with
      i = 0 mod 2^(j+1) receives from worker i + 2^j; the result ends at rank 0.
  R7  The final k values are divided by P after the tree (Eq. 3's average;
      Algorithms 3 and 4 print no division).
  R8  The extra-residual step is a literal add onto the zeroed slot.
  R9  A merged index present in only one operand keeps that operand's value
      bit-for-bit (nothing is added to it).
  R10 Whether a locally selected entry goes back to the residual depends only
      on its INDEX being absent from the global index set (gMask is an index
      mask).
  R11 k-sets are stored index-ascending, indices distinct, uint32.
  R15 Algorithm 1's TopKAllReduce as printed starts its sum from the worker's
      own sparse gradient and slices the gathered arrays with garbled bounds;
      taken literally the own contribution would count twice.  Reading: start
      from a zero vector and add worker g's k entries for g = 0 .. P-1 in that
      order (the printed loop order), then divide by P - which is what the
      comment on the call site states (the average of the P sparse vectors).

Non-finite inputs are outside the method's domain and not supported.

Pins (tests/test_oracle_pins.py): brute force by repeated arg-max on tiny
inputs, library top-k on tie-free inputs, Definition 1 evaluated densely,
P = 2 against the dense sum, shared-support closed form, exact conservation
`sent + residual_new == grad + residual_old`, the restore closed form, and a
hand-worked 4-worker example.  For P > 2 with general inputs the tree is
pinned by composition of pinned merges in the R5 order plus the structural
closed forms (log2 P rounds, P - 1 merges, rank 0 in every round); the paper
prints no numeric example (its worked figures are images).

The pairs of one tree round, and the workers in the local selection and the
restore, are independent of each other: `tree_rounds`, `tree` and `step` take
an optional `map_fn` (default: the builtin `map`) through which those
independent calls are issued, so that a caller may hand in a thread pool's
`map`.  The arithmetic of every call is the same either way.  `topk_allreduce`
is pinned by a per-index Python loop, by exact integer-valued sums, by an
input whose fp32 sum depends on the order, and through P = 2, where its top-k
must equal the tree's result; `dense_topk` by the same brute force and library
top-k as the local selection.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np

_ABS_MASK = np.uint32(0x7FFFFFFF)


def magnitude_keys(v: np.ndarray) -> np.ndarray:
    """R2: |v| as an unsigned integer, `bits(v) & 0x7fffffff`."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    return v.view(np.uint32) & _ABS_MASK


def first_k_by_magnitude(keys: np.ndarray, index: np.ndarray, k: int) -> np.ndarray:
    """The `index` values of the first k entries under the total order
    (key descending, index ascending), returned index-ascending (R1, R11).

    A full sort of one 64-bit composite per entry: high word = key, low word =
    0xFFFFFFFF - index.  Sorted ascending, the LAST k composites are the
    selected ones; the index is read back from the low word.
    """
    n = keys.shape[0]
    assert 0 <= k <= n
    comp = (keys.astype(np.uint64) << np.uint64(32)) | (
        np.uint64(0xFFFFFFFF) - index.astype(np.uint64))
    comp.sort()                                   # full sort; composites are distinct
    chosen = comp[n - k:]
    idx = (np.uint64(0xFFFFFFFF) - (chosen & np.uint64(0xFFFFFFFF))).astype(np.uint32)
    idx.sort()
    return idx


def accumulate(residual: np.ndarray, grad: np.ndarray) -> np.ndarray:
    """Algorithm 4, accumulation: G_i = G_{i-1} + gradient, one fp32 add per element."""
    assert residual.dtype == np.float32 and grad.dtype == np.float32
    return (residual + grad).astype(np.float32)


def local_select(residual: np.ndarray, grad: np.ndarray, k: int
                 ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """The local part of Algorithm 4 for one worker.

    Returns (loc_idx uint32[k] ascending, loc_val float32[k], new residual).
    """
    acc = accumulate(residual, grad)                                 # accumulate
    m = acc.shape[0]
    keys = magnitude_keys(acc)
    loc_idx = first_k_by_magnitude(keys, np.arange(m, dtype=np.uint64), k)  # threshold + mask (R1)
    loc_val = acc[loc_idx].copy()                                     # extract
    new_res = acc.copy()
    new_res[loc_idx] = np.float32(0.0)                                # keep the rest as residual
    return loc_idx, loc_val, new_res


def merge(a_idx: np.ndarray, a_val: np.ndarray, b_idx: np.ndarray, b_val: np.ndarray,
          k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Definition 1: a TOP b, on index-ascending sparse operands.

    Union of the indices (R4); at an index held by both, the two values are
    added with one fp32 add; at an index held by one, its value is copied (R9);
    then the first k under (|v| descending, index ascending); index-ascending out.
    """
    u_idx = np.union1d(a_idx, b_idx).astype(np.uint32)     # sorted, distinct
    assert u_idx.shape[0] >= k
    pa = np.searchsorted(u_idx, a_idx)
    pb = np.searchsorted(u_idx, b_idx)
    in_a = np.zeros(u_idx.shape[0], dtype=bool)
    in_b = np.zeros(u_idx.shape[0], dtype=bool)
    in_a[pa] = True
    in_b[pb] = True
    va = np.zeros(u_idx.shape[0], dtype=np.float32)
    vb = np.zeros(u_idx.shape[0], dtype=np.float32)
    va[pa] = a_val
    vb[pb] = b_val
    both = in_a & in_b
    u_val = np.where(in_a, va, vb).astype(np.float32)       # single-owner: copy
    u_val[both] = (va[both] + vb[both]).astype(np.float32)  # shared: one fp32 add
    out_idx = first_k_by_magnitude(magnitude_keys(u_val), u_idx, k)
    pos = np.searchsorted(u_idx, out_idx)
    return out_idx, u_val[pos].copy()


def tree_rounds(loc_idx: Sequence[np.ndarray], loc_val: Sequence[np.ndarray], k: int,
                map_fn=map) -> List[List[Optional[Tuple[np.ndarray, np.ndarray]]]]:
    """The rounds of Algorithm 3 under R5.  Returns, for each round, the list of
    per-rank current sets after that round (None for ranks that have sent their
    set away and gone idle).  Element [-1][0] is the undivided result.
    The merges of one round are independent and go through `map_fn`."""
    P = len(loc_idx)
    assert P >= 1 and (P & (P - 1)) == 0, "the paper assumes P is a power of two"
    cur: List[Optional[Tuple[np.ndarray, np.ndarray]]] = [
        (np.asarray(loc_idx[w], dtype=np.uint32), np.asarray(loc_val[w], dtype=np.float32))
        for w in range(P)]
    history = []
    n_rounds = P.bit_length() - 1
    for j in range(n_rounds):
        step = 1 << j
        nxt = list(cur)
        receivers = list(range(0, P, 2 * step))

        def one_pair(i, cur=cur, step=step):
            recv = cur[i + step]                      # the partner's set arrives
            mine = cur[i]
            return merge(recv[0], recv[1], mine[0], mine[1], k)    # received TOP own

        for i, merged in zip(receivers, map_fn(one_pair, receivers)):
            nxt[i] = merged
            nxt[i + step] = None                      # the sender goes idle
        cur = nxt                                      # end of the round
        history.append(list(cur))
    if not history:
        history.append(list(cur))
    return history


def tree(loc_idx: Sequence[np.ndarray], loc_val: Sequence[np.ndarray], k: int,
         map_fn=map) -> Tuple[np.ndarray, np.ndarray]:
    """gTopKAllReduce's result as every worker sees it after the broadcast:
    the global index set and the AVERAGED values (R7: sum / P, one fp32 divide)."""
    P = len(loc_idx)
    g_idx, g_sum = tree_rounds(loc_idx, loc_val, k, map_fn)[-1][0]
    g_val = (g_sum / np.float32(P)).astype(np.float32)
    return g_idx.copy(), g_val


def residual_restore(residual: np.ndarray, loc_idx: np.ndarray, loc_val: np.ndarray,
                     g_idx: np.ndarray) -> np.ndarray:
    """Algorithm 4, extra residual, for one worker: locally selected entries whose index
    is not in the global set are added back to the residual (R8, R10)."""
    out = residual.copy()
    globally_kept = np.isin(loc_idx, g_idx)           # gMask at the local indices
    back = ~globally_kept
    out[loc_idx[back]] = (out[loc_idx[back]] + loc_val[back]).astype(np.float32)
    return out


def apply_update(weights: np.ndarray, g_idx: np.ndarray, g_val: np.ndarray, lr) -> np.ndarray:
    """Algorithm 4, model update: W_i = W_{i-1} - eta * G~_i.  G~_i is zero outside g_idx, so
    only those k weights move: one fp32 multiply, then one fp32 subtract."""
    out = weights.copy()
    prod = (np.float32(lr) * g_val.astype(np.float32)).astype(np.float32)
    out[g_idx] = (out[g_idx] - prod).astype(np.float32)
    return out


def dense_mask(g_idx: np.ndarray, m: int) -> np.ndarray:
    """Algorithm 3, after the broadcast: gMask has m entries, 1 at the global indices, 0 elsewhere."""
    mask = np.zeros(m, dtype=np.uint8)
    mask[g_idx] = 1
    return mask


def topk_allreduce(loc_idx: Sequence[np.ndarray], loc_val: Sequence[np.ndarray], m: int
                   ) -> np.ndarray:
    """Algorithm 1, procedure TopKAllReduce (reading R15): a dense m-vector that starts at
    +0.0; worker g's k values are added at worker g's k indices, g = 0 .. P-1 in that
    order, one fp32 add each; then every element is divided by P."""
    P = len(loc_idx)
    dense = np.zeros(m, dtype=np.float32)
    for g in range(P):
        at = loc_idx[g]                      # distinct within a worker
        dense[at] = (dense[at] + loc_val[g]).astype(np.float32)
    return (dense / np.float32(P)).astype(np.float32)


def dense_topk(dense: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Algorithm 2, global selection: the k entries of a dense vector with the largest |v|
    (same R1/R2 rule as the local selection), as an index-ascending sparse k-set."""
    m = dense.shape[0]
    idx = first_k_by_magnitude(magnitude_keys(dense), np.arange(m, dtype=np.uint32), k)
    return idx, dense[idx].copy()


def step(residual: np.ndarray, grad: np.ndarray, k: int, map_fn=map):
    """One full iteration for P workers.  residual, grad: [P][m] float32.

    Returns dict with loc_idx [P][k], loc_val [P][k], g_idx [k], g_val [k],
    residual [P][m] (after the restore) and residual_after_select [P][m].
    The per-worker calls and the pairs of a tree round go through `map_fn`."""
    P, m = grad.shape
    loc_idx = np.empty((P, k), dtype=np.uint32)
    loc_val = np.empty((P, k), dtype=np.float32)
    res_sel = np.empty((P, m), dtype=np.float32)
    selected = map_fn(lambda w: local_select(residual[w], grad[w], k), range(P))
    for w, (li, lv, rs) in enumerate(selected):
        loc_idx[w], loc_val[w], res_sel[w] = li, lv, rs
    g_idx, g_val = tree(list(loc_idx), list(loc_val), k, map_fn)
    res_out = np.empty((P, m), dtype=np.float32)
    restored = map_fn(lambda w: residual_restore(res_sel[w], loc_idx[w], loc_val[w], g_idx),
                      range(P))
    for w, r in enumerate(restored):
        res_out[w] = r
    return {"loc_idx": loc_idx, "loc_val": loc_val, "g_idx": g_idx, "g_val": g_val,
            "residual": res_out, "residual_after_select": res_sel}
