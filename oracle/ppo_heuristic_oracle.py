"""Oracle for the paper's own placement algorithm and its two comparison systems: plain Python, one instance
at a time.  TEST INFRASTRUCTURE ONLY; shares no code with the library.

What is followed (Sec. III-B and Sec. IV of the paper), in the paper's order:
  classes          the transfer sizes are sorted into classes "low" .. "high" (Eq. 5), as many classes as the
                   caller asks for (the evaluation uses 2 .. 20);
  threshold        an edge of the communication graph belongs to the class being matched iff its bandwidth is
                   at or above a threshold (Eq. 8);
  subgraph_k_path  Alg. 2: among the thresholds taken from the edge list sorted by descending bandwidth, the
                   highest one at which the graph of admissible edges still holds a simple path of k nodes
                   (from a given start, to a given end, when those are already fixed), found by bisection; the
                   path's nodes are then taken out of the graph;
  k_path_matching  Alg. 3: classes from the highest down, within a class the runs of consecutive cuts of that
                   class from the longest down; a run of r cuts is matched with a path of r + 1 nodes whose ends
                   are whatever neighbouring runs have already fixed;
  heuristic        Alg. 1 (least sum of transfer sizes under the memory rule) for the cuts, then the matching,
                   then the bottleneck latency of the result by Eq. 2 and Eq. 3;
  random_baseline, joint_baseline   the two comparison systems of Sec. IV.
Arithmetic as everywhere in this repository: binary64 prefix sums of the weights, "fits" is <=, gamma is one
binary32 division (a zero of either sign gives +0).

Readings (the paper leaves these open; the design doc lists them):
  - Classes: equal-width bins between the least and the greatest transfer size of the chain's candidate cuts
    (t[0 .. L-2]); class = min(n_classes - 1, floor((x - lo) / (hi - lo) * n_classes)) in binary64; one class if
    all sizes are equal.
  - The path search of Alg. 2 is the colour-coding method in the paper: a randomised way to find SOME path of k
    nodes.  Here it is a deterministic search that returns the lexicographically smallest such path (depth first
    in increasing node order), with a budget of node expansions after which it reports "none" (the randomised
    method may miss a path too); nodes already used elsewhere in N are not available, the given ends excepted.
  - Thresholds are the distinct bandwidths of the edges among the nodes still available (and the fixed ends).
  - A run both of whose ends are fixed and that has no free node between them (r = 1) is already matched.
  - If some run cannot be matched the result is "no placement" (+inf); `heuristic` then tries again with one
    class fewer, down to one class, as the paper suggests.
  - Random baseline: the random numbers are an input (a list of values in [0, 1)); value x picks item
    floor(x * count).  Joint baseline: ties go to the smaller index; the rest of the chain is taken as the last
    partition as soon as it fits.
"""
import math

import numpy as np

from . import ppo_partition_oracle as PO

KPATH_BUDGET = 20000   # node expansions per path search


def _prefix(m):
    P = [0.0]
    for x in m:
        P.append(P[-1] + float(x))
    return P


def gamma(tv, bw):
    """Eq. 3: one binary32 division; nothing to send takes no time."""
    q = np.float32(tv) / np.float32(bw)
    return np.float32(0.0) if q == 0 else np.float32(q)


def bottleneck(t, B, cuts, nodes):
    """Eq. 2 of a placement: cuts c_1 < ... and the node of every segment."""
    assert len(nodes) == len(cuts) + 1 and len(set(nodes)) == len(nodes)
    beta = np.float32(0.0)
    for s, c in enumerate(cuts, start=1):
        g = gamma(t[c - 1], B[nodes[s - 1]][nodes[s]])
        if g > beta:
            beta = g
    return beta


def transfer_classes(t, sizes, n_classes):
    """Eq. 5: class 0 (lowest) .. n_classes - 1 (highest) of each size, bins of equal width over the chain's sizes."""
    cand = [float(x) for x in t[:-1]] if len(t) > 1 else [0.0]
    lo, hi = min(cand), max(cand)
    out = []
    for x in sizes:
        if hi == lo:
            out.append(n_classes - 1)
        else:
            out.append(min(n_classes - 1, int(math.floor((float(x) - lo) / (hi - lo) * n_classes))))
    return out


def k_path(ok, avail, k, start, end):
    """The lexicographically smallest simple path of k nodes over admissible edges (ok[a][b]).  The first node is
    `start` if given and the last is `end` if given; every other node must be available.  Depth first, nodes in
    increasing order; every node put on the path costs one unit of the budget, and a search that would need more
    than the budget reports None, as does one that finds nothing."""
    n = len(ok)

    def allowed(pos, v):
        if v in path:
            return False
        at_start, at_end = pos == 0 and start is not None, pos == k - 1 and end is not None
        if at_start and v != start:
            return False
        if at_end and v != end:
            return False
        if not at_start and not at_end and not avail[v]:
            return False
        return pos == 0 or bool(ok[path[-1]][v])

    budget = KPATH_BUDGET
    path, nxt = [], [0]
    while True:
        pos = len(path)
        if pos == k:
            return list(path)
        v = nxt[pos]
        while v < n and not allowed(pos, v):
            v += 1
        if v < n:
            if budget == 0:
                return None
            budget -= 1
            nxt[pos] = v + 1
            path.append(v)
            nxt.append(0)
        else:
            nxt.pop()
            if not path:
                return None
            path.pop()


def subgraph_k_path(B, avail, k, start, end):
    """Alg. 2: bisection over the descending list of bandwidths for the highest threshold with a path."""
    n = len(B)
    nodes = [v for v in range(n) if avail[v] or v == start or v == end]
    edge_list = sorted({float(B[a][b]) for a in nodes for b in nodes if a < b}, reverse=True)
    if k == 1 or not edge_list:
        return k_path([[False] * n for _ in range(n)], avail, k, start, end) if k == 1 else None
    low, high, best = 0, len(edge_list), None
    while low < high:
        median = (low + high) // 2
        thr = edge_list[median]
        ok = [[a != b and float(B[a][b]) >= thr for b in range(n)] for a in range(n)]
        result = k_path(ok, avail, k, start, end)
        if result is None:
            low = median + 1
        else:
            high = median
            best = result
    return best


def find_runs(classes, X):
    """maximal runs of consecutive cuts of class X: (first cut index, length)."""
    runs, i = [], 0
    while i < len(classes):
        if classes[i] == X:
            j = i
            while j < len(classes) and classes[j] == X:
                j += 1
            runs.append((i, j - i))
            i = j
        else:
            i += 1
    return runs


def k_path_matching(B, classes, n_classes):
    """Alg. 3: the node of every segment (len(classes) + 1 of them), or None if a run cannot be matched."""
    n, p = len(B), len(classes) + 1
    N = [None] * p
    avail = [True] * n
    if p == 1:
        return [0]            # one segment: the first node (all nodes are alike to the algorithm)
    for X in range(n_classes - 1, -1, -1):
        runs = sorted(find_runs(classes, X), key=lambda r: (-r[1], r[0]))   # longest first, then by position
        for first, length in runs:
            start, end = N[first], N[first + length]
            if start is not None and end is not None and length == 1:
                continue
            path = subgraph_k_path(B, avail, length + 1, start, end)
            if path is None:
                return None
            for i, v in enumerate(path):
                N[first + i] = v
                avail[v] = False
    return N


def heuristic(t, m, kappa, B, n_classes):
    """(beta, segments, cuts, nodes, classes used): the paper's pipeline.  Segments 0 and beta +inf if the chain cannot
    be partitioned or the cluster has fewer nodes than partitions."""
    p, cuts, _ = PO.partition(t, m, kappa)
    n = len(B)
    if p == 0 or p > n:
        return np.float32(np.inf), 0, (), (), 0
    sizes = [t[c - 1] for c in cuts]
    for nc in range(n_classes, 0, -1):
        nodes = k_path_matching(B, transfer_classes(t, sizes, nc), nc)
        if nodes is not None:
            return bottleneck(t, B, cuts, nodes), p, tuple(cuts), tuple(nodes), nc
    return np.float32(np.inf), 0, (), (), 0


def theorem1_bound(t, cuts, B):
    """Theorem 1: the largest chosen transfer size over the largest bandwidth of the cluster."""
    if not cuts:
        return np.float32(0.0)
    n = len(B)
    return gamma(max(float(t[c - 1]) for c in cuts), max(float(B[a][b]) for a in range(n) for b in range(n) if a != b))


def random_baseline(t, m, kappa, B, draws):
    """Sec. IV, first comparison system: again and again a random unused node and a random partition that fits it
    (here: a random number of layers from those that fit, counted from the current layer on).  draws: values in
    [0, 1), two per segment."""
    L, n = len(t), len(B)
    P = _prefix(m)
    free = list(range(n))
    i, d, cuts, nodes = 0, 0, [], []
    while i < L:
        if not free or d + 1 >= len(draws):
            return np.float32(np.inf), 0, (), ()
        node = free.pop(int(float(draws[d]) * len(free)))
        ends = [e for e in range(i + 1, L + 1) if P[e] - P[i] <= float(kappa)]
        if not ends:
            return np.float32(np.inf), 0, (), ()
        e = ends[int(float(draws[d + 1]) * len(ends))]
        d += 2
        nodes.append(node)
        if e < L:
            cuts.append(e)
        i = e
    return bottleneck(t, B, cuts, nodes), len(nodes), tuple(cuts), tuple(nodes)


def joint_baseline(t, m, kappa, B):
    """Sec. IV, second comparison system: partitions by always taking the fitting end with the smallest transfer
    size; nodes by starting somewhere and always moving on over the best link to an unused node; the best start."""
    L, n = len(t), len(B)
    P = _prefix(m)
    cuts, i = [], 0
    while i < L:
        ends = [e for e in range(i + 1, L + 1) if P[e] - P[i] <= float(kappa)]
        if not ends:
            return np.float32(np.inf), 0, (), ()
        e = L if ends[-1] == L else min(ends, key=lambda x: (float(t[x - 1]), x))
        if e < L:
            cuts.append(e)
        i = e
    p = len(cuts) + 1
    if p > n:
        return np.float32(np.inf), 0, (), ()
    best = None
    for first in range(n):
        nodes = [first]
        while len(nodes) < p:
            cur = nodes[-1]
            nxt = max((v for v in range(n) if v not in nodes), key=lambda v: (float(B[cur][v]), -v))
            nodes.append(nxt)
        beta = bottleneck(t, B, cuts, nodes)
        if best is None or beta < best[0]:
            best = (beta, p, tuple(cuts), tuple(nodes))
    return best
