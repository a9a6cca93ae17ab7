"""Oracle for the layer-graph front-end (paper Sec. III-A): plain Python, small graphs only.

TEST INFRASTRUCTURE ONLY; shares no code with the library.  Written from the definitions: the topological
depth LP(v) is the length of the longest path from the source to v; a vertex u is the next candidate
partition point after p iff its depth is unique and EVERY path that leaves p (enumerated one by one here)
reaches u before a deeper vertex; a path that ends before reaching u does not go through it.
Pins (tests/test_dag_frontend.py): a linear chain, a residual block, parallel branches of equal depth, a graph
of two interleaved chains that cannot be partitioned, a dead-end branch: partition points worked out by hand.
"""
from functools import lru_cache


def chain_from_dag(n_vertices, edges, weight, out_size):
    """(t, m, point) as lists; raises ValueError for a graph that is not a DAG with one source."""
    succ = [[] for _ in range(n_vertices)]
    pred = [[] for _ in range(n_vertices)]
    for a, b in edges:
        if not (0 <= a < n_vertices and 0 <= b < n_vertices) or a == b:
            raise ValueError("bad edge")
        succ[a].append(b)
        pred[b].append(a)
    sources = [v for v in range(n_vertices) if not pred[v]]
    if len(sources) != 1:
        raise ValueError("need exactly one source")
    source = sources[0]
    # a cycle: some vertex can reach itself
    state = [0] * n_vertices

    def visit(v):
        if state[v] == 1:
            raise ValueError("cycle")
        if state[v] == 2:
            return
        state[v] = 1
        for u in succ[v]:
            visit(u)
        state[v] = 2

    for v in range(n_vertices):
        visit(v)

    @lru_cache(maxsize=None)
    def lp(v):
        return 0 if v == source else 1 + max(lp(u) for u in pred[v])

    depth = [lp(v) for v in range(n_vertices)]

    def every_path_reaches(p, u):
        def walk(v):
            if v == u:
                return True
            if depth[v] > depth[u] or not succ[v]:
                return False
            return all(walk(x) for x in succ[v])
        return all(walk(x) for x in succ[p]) if succ[p] else False

    points = [source]
    for d in range(1, max(depth) + 1):
        here = [v for v in range(n_vertices) if depth[v] == d]
        if len(here) == 1 and every_path_reaches(points[-1], here[0]):
            points.append(here[0])
    t, m, point = [], [], []
    lower = -1
    for p in points:
        group = [v for v in range(n_vertices) if lower < depth[v] <= depth[p]]
        m.append(sum(float(weight[v]) for v in group))
        t.append(float(out_size[p]))
        point.append(p)
        lower = depth[p]
    tail = [v for v in range(n_vertices) if depth[v] > lower]
    if tail:
        m.append(sum(float(weight[v]) for v in tail))
        t.append(0.0)
        point.append(-1)
    return t, m, point
