"""The layer-graph front-end (ppo_chain_from_dag, host code; paper Sec. III-A): hand-worked partition points,
and the library against the plain-Python oracle on random layer graphs."""
import ctypes as C

import numpy as np
import pytest

from oracle import ppo_dag_oracle as DO
from paper_2210_12219_amd import binding

ROUTES = {
    "oracle": lambda n, e, w, o: tuple(np.asarray(x) for x in DO.chain_from_dag(n, e, w, o)),
    "library": lambda n, e, w, o: binding.ppo_chain_from_dag(n, e, w, o),
}


def sizes(n):
    return np.arange(1, n + 1, dtype=np.float32), 10.0 * np.arange(1, n + 1, dtype=np.float32)


@pytest.mark.parametrize("route", ROUTES)
def test_hand_worked_graphs(route):
    f = ROUTES[route]
    # a plain chain: every layer is a partition point
    w, o = sizes(5)
    t, m, p = f(5, [(0, 1), (1, 2), (2, 3), (3, 4)], w, o)
    assert list(p) == [0, 1, 2, 3, 4] and list(m) == list(w) and list(t) == list(o)
    # a residual block 0 -> 1 -> 2 -> 3 with the shortcut 0 -> 3, then 4: the shortcut passes 1 and 2 by
    t, m, p = f(5, [(0, 1), (1, 2), (2, 3), (0, 3), (3, 4)], w, o)
    assert list(p) == [0, 3, 4] and list(m) == [1.0, 2.0 + 3.0 + 4.0, 5.0] and list(t) == [10.0, 40.0, 50.0]
    # two branches of equal depth: neither 1 nor 2 has its depth to itself
    w4, o4 = sizes(4)
    t, m, p = f(4, [(0, 1), (0, 2), (1, 3), (2, 3)], w4, o4)
    assert list(p) == [0, 3] and list(m) == [1.0, 9.0] and list(t) == [10.0, 40.0]
    # two interleaved chains (every depth is shared, two outputs): nothing but the source, the rest is one layer
    w7, o7 = sizes(7)
    edges = [(0, 1), (0, 2), (1, 3), (2, 4), (1, 4), (2, 3), (3, 5), (4, 6), (3, 6), (4, 5)]
    t, m, p = f(7, edges, w7, o7)
    assert list(p) == [0, -1] and list(m) == [1.0, float(sum(range(2, 8)))] and list(t) == [10.0, 0.0]
    # a side output 1 -> 4 that ends: 3 has its depth to itself, but the path 1 -> 4 never reaches it
    t, m, p = f(5, [(0, 1), (1, 2), (2, 3), (1, 4)], w, o)
    assert list(p) == [0, 1, -1] and list(m) == [1.0, 2.0, 3.0 + 4.0 + 5.0] and list(t) == [10.0, 20.0, 0.0]
    # a single layer
    t, m, p = f(1, [], np.array([7.0], np.float32), np.array([3.0], np.float32))
    assert list(p) == [0] and list(m) == [7.0] and list(t) == [3.0]
    # a longer shortcut: 0 -> 1 -> 2 -> 3 -> 4 -> 5 with 1 -> 4: points 0, 1, 4, 5
    w6, o6 = sizes(6)
    t, m, p = f(6, [(0, 1), (1, 2), (2, 3), (3, 4), (4, 5), (1, 4)], w6, o6)
    assert list(p) == [0, 1, 4, 5] and list(m) == [1.0, 2.0, 3.0 + 4.0 + 5.0, 6.0]


def random_layer_graph(rng, n):
    """A DAG on 0..n-1, vertex 0 the only source: mostly a chain, with shortcuts, branches and side outputs,
    vertices relabelled at random (the library must not rely on their order)."""
    edges = set()
    for v in range(1, n):
        edges.add((v - 1, v) if rng.random() < 0.8 else (int(rng.integers(0, v)), v))
    for _ in range(int(rng.integers(0, max(1, n // 3) + 1))):
        a = int(rng.integers(0, n - 1))
        edges.add((a, int(rng.integers(a + 1, n))))
    relabel = np.concatenate([[0], 1 + rng.permutation(n - 1)])
    return [(int(relabel[a]), int(relabel[b])) for a, b in sorted(edges)]


def test_library_equals_oracle_on_random_graphs():
    rng = np.random.default_rng(5)
    seen_points = 0
    for case in range(400):
        n = int(rng.integers(2, 15))
        edges = random_layer_graph(rng, n)
        w = rng.uniform(0.1, 50.0, n).astype(np.float32)
        o = rng.uniform(0.1, 20.0, n).astype(np.float32)
        t0, m0, p0 = (np.asarray(x) for x in DO.chain_from_dag(n, edges, w, o))
        t1, m1, p1 = binding.ppo_chain_from_dag(n, edges, w, o)
        assert list(p0) == list(p1), (case, edges)
        assert np.array_equal(t0.astype(np.float32), t1)
        assert np.array_equal(m0.astype(np.float32), m1)   # the oracle adds in binary64 in vertex order too
        assert abs(float(m1.sum()) - float(w.sum())) <= 1e-3 * float(w.sum())   # every layer lands in the chain once
        seen_points += len(p1)
    assert seen_points > 3 * 400   # the graphs are not all trivial


def test_bad_graphs_are_refused():
    lib = binding.load()
    i32 = lambda a: np.ascontiguousarray(a, dtype=np.int32)
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    ptr = lambda a: C.c_void_p(a.ctypes.data)

    def call(n, edges, cap=16):
        e = i32(edges).reshape(-1, 2)
        src, dst = i32(e[:, 0]), i32(e[:, 1])
        w, o = f32(np.ones(max(n, 1))), f32(np.ones(max(n, 1)))
        t, m, p, L = f32(np.zeros(cap)), f32(np.zeros(cap)), i32(np.zeros(cap)), C.c_int32(0)
        rc = lib.ppo_chain_from_dag(n, len(src), ptr(src), ptr(dst), ptr(w), ptr(o), cap, ptr(t), ptr(m), ptr(p),
                                    C.cast(C.byref(L), C.c_void_p))
        return rc, L.value

    assert call(3, [(0, 1), (1, 2)]) == (binding.PPO_OK, 3)
    assert call(3, [(0, 1), (1, 2), (2, 1)])[0] == binding.PPO_EINVAL        # a cycle
    assert call(3, [(0, 2), (1, 2)])[0] == binding.PPO_EINVAL                # two sources
    assert call(3, [(0, 1), (1, 3)])[0] == binding.PPO_EINVAL                # vertex out of range
    assert call(3, [(0, 1), (1, 1)])[0] == binding.PPO_EINVAL                # self loop
    assert call(0, [])[0] == binding.PPO_EINVAL
    assert call(4, [(0, 1), (1, 2), (2, 3)], cap=2) == (binding.PPO_ENOSPC, 4)
    for bad in ([(0, 1), (1, 2), (2, 1)], [(0, 2), (1, 2)]):
        with pytest.raises(ValueError):
            DO.chain_from_dag(3, bad, np.ones(3), np.ones(3))


def test_a_very_long_layer_graph_needs_no_deep_recursion():
    """300,000 residual blocks in a row, and one shortcut from the source past all of them: the walk from a
    partition point towards a candidate passes every vertex in between."""
    blocks = 300_000
    edges, v = [], 0
    for _ in range(blocks):
        edges += [(v, v + 1), (v + 1, v + 2), (v, v + 2)]
        v += 2
    n = v + 1
    w = np.ones(n, np.float32)
    o = np.full(n, 2.0, np.float32)
    t, m, p = binding.ppo_chain_from_dag(n, edges, w, o)
    assert len(p) == blocks + 1 and list(p[:3]) == [0, 2, 4] and (m[1:] == 2.0).all() and m[0] == 1.0
    edges.append((0, n - 1))              # now nothing but the source and the last vertex is a point
    t, m, p = binding.ppo_chain_from_dag(n, edges, w, o)
    assert list(p) == [0, n - 1] and m[1] == np.float32(n - 1)
