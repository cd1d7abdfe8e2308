"""Property tests of the CPU oracle on many small random inputs (hypothesis, derandomised):
each property follows from the paper's definitions alone and is checked with code that
shares nothing with the oracle's implementation (pure-Python loops on exact float images)."""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import gtopk_oracle as orc

SETTINGS = dict(max_examples=120, deadline=None, derandomize=True)

# values that make ties, signed zeros and denormals common
VALUE = st.one_of(
    st.sampled_from([0.0, -0.0, 1.0, -1.0, 0.5, -0.5, 2.0, -2.0, 1e-40, -1e-40, 3.5, -3.5]),
    st.floats(min_value=-8, max_value=8, allow_nan=False, width=32),
)


def f32(x):
    return np.float32(x)


def key(x):
    return int(np.array([x], dtype=np.float32).view(np.uint32)[0]) & 0x7FFFFFFF


def first_k(pairs, k):
    """pairs: list of (index, value); the first k under (|v| descending, index ascending)."""
    order = sorted(pairs, key=lambda p: (-key(p[1]), p[0]))
    return sorted(order[:k], key=lambda p: p[0])


@settings(**SETTINGS)
@given(st.lists(st.tuples(VALUE, VALUE), min_size=1, max_size=40), st.data())
def test_local_select_is_the_definition(rows, data):
    res = np.array([r[0] for r in rows], dtype=np.float32)
    grad = np.array([r[1] for r in rows], dtype=np.float32)
    m = len(rows)
    k = data.draw(st.integers(1, m))
    idx, val, new_res = orc.local_select(res, grad, k)
    acc = [f32(res[i] + grad[i]) for i in range(m)]
    want = first_k(list(enumerate(acc)), k)
    assert idx.tolist() == [p[0] for p in want]
    assert val.view(np.uint32).tolist() == [int(np.array([p[1]]).view(np.uint32)[0]) for p in want]
    chosen = set(idx.tolist())
    for i in range(m):
        expect = f32(0.0) if i in chosen else acc[i]
        assert new_res[i].view(np.uint32) == np.array([expect]).view(np.uint32)[0]


def sparse_set(draw, m, k):
    idx = sorted(draw(st.lists(st.integers(0, m - 1), min_size=k, max_size=k, unique=True)))
    val = [draw(VALUE) for _ in range(k)]
    return np.array(idx, dtype=np.uint32), np.array(val, dtype=np.float32)


@settings(**SETTINGS)
@given(st.data())
def test_merge_is_definition_1(data):
    m = data.draw(st.integers(1, 30))
    k = data.draw(st.integers(1, m))
    a_idx, a_val = sparse_set(data.draw, m, k)
    b_idx, b_val = sparse_set(data.draw, m, k)
    o_idx, o_val = orc.merge(a_idx, a_val, b_idx, b_val, k)
    da = dict(zip(a_idx.tolist(), a_val.tolist()))
    db = dict(zip(b_idx.tolist(), b_val.tolist()))
    union = []
    for i in sorted(set(da) | set(db)):
        if i in da and i in db:
            union.append((i, f32(f32(da[i]) + f32(db[i]))))
        else:
            union.append((i, f32(da[i] if i in da else db[i])))
    want = first_k(union, k)
    assert o_idx.tolist() == [p[0] for p in want]
    assert o_val.view(np.uint32).tolist() == [int(np.array([p[1]]).view(np.uint32)[0]) for p in want]


@settings(**SETTINGS)
@given(st.data())
def test_tree_is_nested_merges_then_average(data):
    P = data.draw(st.sampled_from([1, 2, 4, 8]))
    m = data.draw(st.integers(2, 24))
    k = data.draw(st.integers(1, m))
    sets = [sparse_set(data.draw, m, k) for _ in range(P)]
    g_idx, g_val = orc.tree([s[0] for s in sets], [s[1] for s in sets], k)
    cur = list(sets)
    while len(cur) > 1:                       # pairs (0,1), (2,3), ... of the survivors
        cur = [orc.merge(cur[i][0], cur[i][1], cur[i + 1][0], cur[i + 1][1], k)
               for i in range(0, len(cur), 2)]
    assert g_idx.tolist() == cur[0][0].tolist()
    assert g_val.view(np.uint32).tolist() == (cur[0][1] / f32(P)).astype(np.float32).view(np.uint32).tolist()


@settings(**SETTINGS)
@given(st.data())
def test_restore_and_allreduce(data):
    P = data.draw(st.integers(1, 5))
    m = data.draw(st.integers(1, 24))
    k = data.draw(st.integers(1, m))
    sets = [sparse_set(data.draw, m, k) for _ in range(P)]
    dense = orc.topk_allreduce([s[0] for s in sets], [s[1] for s in sets], m)
    for i in range(m):
        acc = f32(0.0)
        for idx, val in sets:
            for t in range(k):
                if int(idx[t]) == i:
                    acc = f32(acc + val[t])
        assert dense[i].view(np.uint32) == np.array([f32(acc / f32(P))]).view(np.uint32)[0]
    g_idx, _ = orc.dense_topk(dense, k)
    residual = np.array([data.draw(VALUE) for _ in range(m)], dtype=np.float32)
    out = orc.residual_restore(residual, sets[0][0], sets[0][1], g_idx)
    inside = set(g_idx.tolist())
    for i in range(m):
        expect = residual[i]
        for t in range(k):
            if int(sets[0][0][t]) == i and i not in inside:
                expect = f32(residual[i] + sets[0][1][t])
        assert out[i].view(np.uint32) == np.array([expect]).view(np.uint32)[0]
