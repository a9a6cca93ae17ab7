"""Pins of the oracle of the paper's own placement algorithm (oracle/ppo_heuristic_oracle.py; Sec. III-B Eq. 5 and
Eq. 8, Alg. 2, Alg. 3; Sec. IV comparison systems): examples worked by hand, brute force over every path, and what
the paper itself states (Theorem 1 is a lower bound for the chosen cuts; nothing beats the exact optimum)."""
import itertools

import numpy as np
import pytest

from oracle import ppo_cluster_oracle as CO
from oracle import ppo_heuristic_oracle as H
from paper_2210_12219_amd import workloads as W


def sym(n, entries, fill=1.0):
    B = np.full((n, n), fill, np.float32)
    np.fill_diagonal(B, 0)
    for (a, b), v in entries.items():
        B[a, b] = B[b, a] = v
    return B


def test_transfer_size_classes_by_hand():
    """Eq. 5 with three classes over sizes 0 .. 9: bins [0,3), [3,6), [6,9]; the greatest size is in the top class."""
    t = np.array([0, 9, 4, 2, 6, 3, 8.99, 5.99, 7], np.float32)     # the last entry is not a candidate cut
    assert H.transfer_classes(t, [0, 2.9, 3, 5.99, 6, 8.99, 9], 3) == [0, 0, 1, 1, 2, 2, 2]
    assert H.transfer_classes(t, [4.4, 4.5], 2) == [0, 1]
    assert H.transfer_classes(np.array([5, 5, 5, 1], np.float32), [5, 5], 4) == [3, 3]          # all sizes equal
    assert H.transfer_classes(t, [1, 8], 1) == [0, 0]


def test_path_search_by_hand():
    """Five nodes; admissible edges 0-1, 1-2, 2-3, 0-3, 3-4."""
    ok = [[False] * 5 for _ in range(5)]
    for a, b in ((0, 1), (1, 2), (2, 3), (0, 3), (3, 4)):
        ok[a][b] = ok[b][a] = True
    free = [True] * 5
    assert H.k_path(ok, free, 3, None, None) == [0, 1, 2]                 # the smallest sequence
    assert H.k_path(ok, free, 5, None, None) == [0, 1, 2, 3, 4]
    # ending at 4 with four nodes: nothing starts at 0 (0-1-2-3 ends at 3, 0-3-4 is too short); from 1: 1-0-3-4
    assert H.k_path(ok, free, 4, None, 4) == [1, 0, 3, 4]
    assert H.k_path(ok, free, 3, 4, None) == [4, 3, 0]                    # from 4: 4-3-0 before 4-3-2
    assert H.k_path(ok, free, 3, 1, 3) == [1, 0, 3]                       # both ends fixed: via 0 before via 2
    used = [True, True, False, True, True]                                # node 2 is taken
    assert H.k_path(ok, used, 4, None, None) == [1, 0, 3, 4]
    assert H.k_path(ok, used, 5, None, None) is None
    # fixed ends are themselves not "available" (they already sit in N) and may only close the path
    taken = [False, True, True, False, True]
    assert H.k_path(ok, taken, 4, 0, 3) == [0, 1, 2, 3]
    assert H.k_path(ok, taken, 2, 0, 3) == [0, 3]
    assert H.k_path(ok, free, 1, None, None) == [0] and H.k_path(ok, taken, 1, None, None) == [1]


def test_path_search_budget(monkeypatch):
    """A complete graph of 8 nodes and a path of 8: found with 8 expansions; with a budget of 7 the search gives up."""
    ok = [[a != b for b in range(8)] for a in range(8)]
    monkeypatch.setattr(H, "KPATH_BUDGET", 8)
    assert H.k_path(ok, [True] * 8, 8, None, None) == list(range(8))
    monkeypatch.setattr(H, "KPATH_BUDGET", 7)
    assert H.k_path(ok, [True] * 8, 8, None, None) is None


def best_path_by_brute_force(B, avail, k, start, end):
    """Every sequence of k distinct nodes: the greatest least-bandwidth, and the smallest sequence that reaches it."""
    n = len(B)
    best = None
    for seq in itertools.permutations(range(n), k):
        if start is not None and seq[0] != start:
            continue
        if end is not None and seq[-1] != end:
            continue
        inner = [v for i, v in enumerate(seq) if not ((i == 0 and start is not None) or (i == k - 1 and end is not None))]
        if not all(avail[v] for v in inner):
            continue
        width = min(float(B[a][b]) for a, b in zip(seq, seq[1:])) if k > 1 else 0.0
        key = (-width, seq)
        if best is None or key < best:
            best = key
    return None if best is None else list(best[1])


def test_alg2_finds_the_widest_path_and_the_smallest_such():
    """Alg. 2's bisection ends at the highest threshold that still admits a path of k nodes, i.e. at the path whose
    weakest link is strongest; among those the search returns the smallest sequence.  Brute force over all sequences."""
    rng = np.random.default_rng(8)
    for trial in range(120):
        n = int(rng.integers(2, 7))
        B = np.zeros((n, n), np.float32)
        iu = np.triu_indices(n, 1)
        B[iu] = rng.integers(1, 6, len(iu[0])) if trial % 2 else np.exp(rng.uniform(0, 4, len(iu[0])))
        B = B + B.T
        avail = [bool(x) for x in rng.integers(0, 4, n) > 0]
        k = int(rng.integers(1, n + 1))
        start = int(rng.integers(0, n)) if trial % 3 == 0 else None
        end = int(rng.integers(0, n)) if trial % 5 == 0 else None
        if start is not None and start == end and k > 1:
            end = None
        fixed = [v for v in (start, end) if v is not None]
        av = [a and v not in fixed for v, a in enumerate(avail)]
        want = best_path_by_brute_force(B, av, k, start, end)
        if k == 1 and start is not None and end is not None and start != end:
            want = None
        got = H.subgraph_k_path(B, av, k, start, end)
        assert got == want, (trial, n, k, start, end, got, want)


def test_alg3_matching_by_hand():
    """Six nodes, five segments; the cuts' classes, high to low: cut 1 and 2 high, cut 0 low, cut 3 low.
    Bandwidths: 0-1 9, 1-2 8, 2-3 7 are the best links; everything else 1 except 3-4 3, 2-5 2, 0-5 4.
    High run (cuts 1, 2: nodes N1 N2 N3): the widest path of three nodes is 0-1-2 (weakest link 8).
    Low runs, equally long, by position: cut 0 (N0 then N1 = 0): best link into node 0 from a free node: 0-5 (4):
    N0 = 5.  Cut 3 (N3 = 2 then N4): best free neighbour of 2: node 3 (7).  N = 5 0 1 2 3."""
    B = sym(6, {(0, 1): 9, (1, 2): 8, (2, 3): 7, (3, 4): 3, (2, 5): 2, (0, 5): 4})
    assert H.k_path_matching(B, [0, 2, 2, 0], 3) == [5, 0, 1, 2, 3]
    # with one class the whole chain is one run: the widest path of five nodes, smallest sequence
    one = H.k_path_matching(B, [0, 0, 0, 0], 1)
    assert one == best_path_by_brute_force(B, [True] * 6, 5, None, None)
    # more partitions than nodes left for a run: no placement
    assert H.k_path_matching(sym(3, {}), [1, 1, 0, 0], 2) is None
    assert H.k_path_matching(B, [], 3) == [0]


def test_comparison_systems_by_hand():
    t = np.array([5, 1, 4, 2, 9], np.float32)
    m = np.array([2, 2, 2, 2, 2], np.float32)
    B = sym(4, {(0, 1): 2, (1, 2): 4, (0, 2): 8, (2, 3): 1, (0, 3): 3, (1, 3): 5})
    # joint baseline, capacity 4 (two layers at most): from layer 0 the ends 1 (t 5) and 2 (t 1): 2; from 2 the ends
    # 3 (t 4) and 4 (t 2): 4; then layer 4 alone.  Cuts 2, 4: sizes 1 and 2.  Node paths by best link: from 0:
    # 0-2 (8), 2-1 (4): max(1/8, 2/4) = 0.5; from 1: 1-3 (5), 3-0 (3): max(0.2, 2/3); from 2: 2-0, 0-3 (3):
    # max(1/8, 2/3); from 3: 3-1 (5), 1-2 (4): max(0.2, 0.5) = 0.5.  Best 0.5, first reached from node 0.
    beta, p, cuts, nodes = H.joint_baseline(t, m, 4.0, B)
    assert float(beta) == 0.5 and p == 3 and cuts == (2, 4) and nodes == (0, 2, 1)
    # random baseline: draws (node, size) per segment.  0.6 of four nodes: node 2; 0.9 of the two fitting ends: 2.
    # 0.0 of three: node 0; 0.0 of ends (3, 4): 3.  0.5 of two: node 3 (free = 1, 3); 0.99 of ends (4, 5): 5, done.
    beta, p, cuts, nodes = H.random_baseline(t, m, 4.0, B, [0.6, 0.9, 0.0, 0.0, 0.5, 0.99])
    assert p == 3 and cuts == (2, 3) and nodes == (2, 0, 3)
    assert beta == max(np.float32(1) / np.float32(8), np.float32(4) / np.float32(3))
    assert np.isinf(H.random_baseline(t, m, 1.0, B, [0.1] * 10)[0])            # nothing fits a node
    assert np.isinf(H.joint_baseline(t, m, 2.0, B)[0])                          # five partitions, four nodes


def test_heuristic_against_the_bound_and_the_exact_optimum():
    """What the paper states about its own algorithm, on paper-shaped clusters: Theorem 1 is a lower bound for the
    cuts chosen; and no placement, the heuristic's and the comparison systems' included, beats the exact optimum."""
    seen_gap = 0
    for n, cap in ((5, 32), (6, 24), (8, 32), (10, 16), (10, 32)):
        w = W.cluster_geometric(n, cap, n_inst=5, seed=40 + n)
        for i in range(w.n_inst):
            for nc in (2, 5, 8):
                beta, p, cuts, nodes, used = H.heuristic(w.t[i], w.m[i], w.M[i][0], w.B[i], nc)
                exact = CO.subset_dp(w.t[i], w.m[i], w.M[i], w.B[i])[0]
                assert np.isfinite(beta) and 1 <= used <= nc and len(nodes) == p == len(cuts) + 1
                assert beta == H.bottleneck(w.t[i], w.B[i], cuts, nodes)
                assert H.theorem1_bound(w.t[i], cuts, w.B[i]) <= beta
                assert exact <= beta
                seen_gap += bool(exact < beta)
            joint = H.joint_baseline(w.t[i], w.m[i], w.M[i][0], w.B[i])[0]
            rnd = H.random_baseline(w.t[i], w.m[i], w.M[i][0], w.B[i], np.random.default_rng(i).random(40))[0]
            assert exact <= joint and exact <= rnd
    assert seen_gap >= 10       # the exact search does find better placements than the heuristic
