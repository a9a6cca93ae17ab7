"""Pins for the CPU oracle: facts fixed by the paper and by the mathematics, none of them
produced by the oracle itself (and none by the HIP path)."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import ppo_oracle as O
from paper_2210_12219_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ROUTES = {
    "bruteforce": lambda t, m, M, B: O.bruteforce(t, m, M, B),
    "exhaustive": lambda t, m, M, B: O.exhaustive(t, m, M, B)[:3],
    "subset_dp": lambda t, m, M, B: O.subset_dp(t, m, M, B),
}


def bits(x):
    return np.asarray(x, dtype=np.float32).view(np.uint32)


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                key, val = line.split()
                out[key] = val
    return out


def const_bandwidth(k, b):
    B = np.full((k, k), b, dtype=np.float32)
    np.fill_diagonal(B, 0)
    return B


@pytest.mark.parametrize("route", ROUTES)
def test_worked_example_from_the_paper(route):
    """Sec. I: 10.2 Mbit over 6 Mbps is about 1.7 s."""
    g = read_golden("worked_example.txt")
    t = np.array([float(g["t_mbit"]), 3.0], np.float32)
    m = np.array([1.0, 1.0], np.float32)
    M = np.array([5.0, 5.0], np.float32)
    B = const_bandwidth(2, float(g["bandwidth_mbps"]))
    beta, cuts, order = ROUTES[route](t, m, M, B)
    assert int(bits(beta)[0]) == int(g["beta_bits"], 16)
    assert abs(float(beta[0]) - float(g["paper_seconds"])) < 1e-6
    assert cuts.tolist() == [[1]] and order.tolist() == [[0, 1]]


def test_rank_is_the_lexicographic_index():
    for k in range(1, 8):
        for r, p in enumerate(itertools.permutations(range(k))):
            assert O.rank(p) == r
            assert tuple(O.unrank(r, k)) == p


@pytest.mark.parametrize("k", [8, 10, 11, 12])
def test_rank_unrank_large_k(k):
    rng = np.random.default_rng(k)
    kf = math.factorial(k)
    assert O.unrank(0, k).tolist() == list(range(k))
    assert O.unrank(kf - 1, k).tolist() == list(range(k))[::-1]
    for r in rng.integers(0, kf - 1, 200):
        r = int(r)
        a, b = tuple(O.unrank(r, k)), tuple(O.unrank(r + 1, k))
        assert sorted(a) == list(range(k))
        assert a < b                      # lexicographic order of tuples
        assert O.rank(a) == r
        # b is the immediate successor: they share a prefix, then b's suffix is the smallest
        # arrangement that is larger (checked via the standard successor construction in itertools terms)
        i = next(j for j in range(k) if a[j] != b[j])
        assert sorted(a[i:]) == sorted(b[i:])
        assert list(b[i + 1:]) == sorted(b[i + 1:])
        assert b[i] == min(x for x in a[i + 1:] if x > a[i])
        assert list(a[i + 1:]) == sorted(a[i + 1:], reverse=True)


@pytest.mark.parametrize("route", ROUTES)
def test_single_node(route):
    """k = 1: no link is crossed, beta = 0 iff the whole model fits."""
    t = np.array([3, 1, 4, 1, 5], np.float32)
    m = np.array([1, 2, 3, 4, 5], np.float32)
    B = np.zeros((1, 1), np.float32)
    beta, cuts, order = ROUTES[route](t, m, np.array([15.0], np.float32), B)
    assert bits(beta)[0] == 0 and order.tolist() == [[0]] and cuts.shape == (1, 0)
    beta, cuts, order = ROUTES[route](t, m, np.array([14.99], np.float32), B)
    assert np.isinf(beta[0]) and order.tolist() == [[-1]]


@pytest.mark.parametrize("route", ROUTES)
def test_two_nodes_closed_form(route):
    """k = 2: beta* = min over the cut i and both orderings with both halves fitting of t[i-1]/B01."""
    rng = np.random.default_rng(7)
    for _ in range(200):
        L = int(rng.integers(2, 12))
        w = W.random_instances(int(rng.integers(1 << 30)), 1, L, 2, capacity_factor=float(rng.uniform(0.9, 1.6)),
                               quantised=bool(rng.integers(2)))
        t, m, M, B = w.t[0], w.m[0], w.M[0], w.B[0]
        P = np.concatenate([[0.0], np.cumsum(m.astype(np.float64))])
        best = None
        for a, b in ((0, 1), (1, 0)):                     # rank order
            for i in range(1, L):
                if P[i] <= float(M[a]) and P[L] - P[i] <= float(M[b]):
                    q = np.float32(t[i - 1]) / np.float32(B[a, b])
                    if best is None or q < best[0]:
                        best = (q, [a, b], i)
        beta, cuts, order = ROUTES[route](t, m, M, B)
        if best is None:
            assert np.isinf(beta[0]) and cuts.tolist() == [[-1]] and order.tolist() == [[-1, -1]]
        else:
            assert bits(beta)[0] == bits(best[0]) and order[0].tolist() == best[1] and cuts[0, 0] == best[2]


@pytest.mark.parametrize("route", ["exhaustive", "subset_dp"])
def test_no_memory_limit_constant_bandwidth(route):
    """With ample memory and one bandwidth b, beta* is the (k-1)-th smallest of t[0..L-2] over b,
    the identity ordering (rank 0) wins, and the cuts sit after the k-1 smallest values
    (unique here because the values are distinct)."""
    rng = np.random.default_rng(11)
    for _ in range(60):
        L = int(rng.integers(3, 15))
        k = int(rng.integers(2, min(L, 5) + 1))
        t = rng.permutation(np.arange(1, L + 1)).astype(np.float32) * np.float32(0.37)
        m = rng.uniform(1, 2, L).astype(np.float32)
        M = np.full(k, 1e6, np.float32)
        b = np.float32(rng.uniform(1, 9))
        beta, cuts, order = ROUTES[route](t, m, M, const_bandwidth(k, b))
        smallest = np.sort(t[:L - 1])[:k - 1]
        assert bits(beta)[0] == bits(smallest[-1] / b)
        assert order[0].tolist() == list(range(k))
        assert cuts[0].tolist() == sorted(int(np.where(t == v)[0][0]) + 1 for v in smallest)


def test_homogeneous_memory_constant_bandwidth_is_ordering_independent():
    """The paper's own setting (Sec. I: all nodes take the smallest capacity): with one bandwidth as well,
    every ordering has the same beta."""
    w = W.random_instances(5, 1, 10, 4)
    M = np.full(4, float(w.m[0].sum()) * 0.8, np.float32)
    out, _ = O.eval_orderings(w.t[0], w.m[0], M, const_bandwidth(4, 3.0), 0, 24)
    assert len(set(bits(out).tolist())) == 1 and np.isfinite(out[0])
    beta, cuts, order, _ = O.exhaustive(w.t[0], w.m[0], M, const_bandwidth(4, 3.0))
    assert order[0].tolist() == [0, 1, 2, 3] and bits(beta)[0] == bits(out)[0]


def test_three_routes_agree_on_small_instances():
    """Brute force over every (cut vector, permutation) pair is the definition itself; the per-ordering DP
    and the subset DP must reproduce beta, the ordering (rule T1) and the cuts (rule T2) exactly.
    Quantised instances force equal latencies and capacities that are hit exactly."""
    n_checked = n_inf = n_ties = 0
    for seed in range(60):
        rng = np.random.default_rng(1000 + seed)
        L = int(rng.integers(2, 10))
        k = int(rng.integers(1, min(L, 4) + 1))
        w = W.random_instances(seed, 60, L, k, capacity_factor=float(rng.uniform(1.0, 1.8)),
                               quantised=bool(seed % 2))
        ref = O.bruteforce(w.t, w.m, w.M, w.B)
        ex = O.exhaustive(w.t, w.m, w.M, w.B, n_threads=2)[:3]
        sub = O.subset_dp(w.t, w.m, w.M, w.B, n_threads=2)
        for got in (ex, sub):
            assert np.array_equal(bits(ref[0]), bits(got[0]))
            assert np.array_equal(ref[1], got[1])
            assert np.array_equal(ref[2], got[2])
        n_checked += w.n_inst
        n_inf += int(np.isinf(ref[0]).sum())
        if seed % 2 and k >= 2:
            for j in range(0, w.n_inst, 10):
                per, _ = O.eval_orderings(w.t[j], w.m[j], w.M[j], w.B[j], 0, math.factorial(k))
                n_ties += int((bits(per) == bits(ref[0][j])).sum() > 1)
    assert n_checked == 3600 and 50 < n_inf < n_checked - 500 and n_ties > 20


def test_capacity_hit_exactly_counts_as_fitting():
    """The memory rule reads 'within the capacity' (Sec. III-B, text under Eq. 6): equality fits."""
    t = np.array([1, 2, 3, 4], np.float32)
    m = np.array([2, 3, 3, 1], np.float32)
    B = const_bandwidth(2, 1.0)
    for route in ROUTES.values():
        beta, cuts, order = route(t, m, np.array([5.0, 5.0], np.float32), B)
        assert float(beta[0]) == 2.0 and cuts.tolist() == [[2]]
        beta, cuts, order = route(t, m, np.array([4.999, 5.0], np.float32), B)   # node 0 cannot take [0,2)
        assert float(beta[0]) == 2.0 and order.tolist() == [[1, 0]]
        beta, cuts, order = route(t, m, np.array([4.999, 4.999], np.float32), B)
        assert np.isinf(beta[0])


def test_memory_rule_is_taken_in_binary64():
    """Segment sizes are sums of binary32 weights taken in binary64 and compared there with the capacity:
    2^24 + 1 exceeds a capacity of 2^24, although it rounds to 2^24 in binary32 (by hand, both ways)."""
    big = np.float32(2.0 ** 24)
    for route in ROUTES.values():
        # one node: the whole model must fit it
        beta, _, order = route(np.array([1, 1], np.float32), np.array([big, 1], np.float32),
                               np.array([big], np.float32), const_bandwidth(1, 1.0))
        assert np.isinf(beta[0]) and order.tolist() == [[-1]]
        beta, _, _ = route(np.array([1, 1, 1], np.float32), np.array([big, 1, 1], np.float32),
                           np.array([big], np.float32), const_bandwidth(1, 1.0))   # 2^24 + 1 + 1, summed in order
        assert np.isinf(beta[0])
        beta, _, _ = route(np.array([1, 1], np.float32), np.array([big, 1], np.float32),
                           np.array([big + np.float32(2)], np.float32), const_bandwidth(1, 1.0))
        assert float(beta[0]) == 0.0
        # two nodes: neither cut leaves both segments within 2^24
        t = np.array([3, 5, 7], np.float32)
        m = np.array([1, big, 1], np.float32)
        beta, cuts, _ = route(t, m, np.array([big, big], np.float32), const_bandwidth(2, 1.0))
        assert np.isinf(beta[0]) and cuts.tolist() == [[-1]]
        beta, cuts, _ = route(t, m, np.array([big, big + np.float32(2)], np.float32), const_bandwidth(2, 1.0))
        assert float(beta[0]) == 3.0 and cuts.tolist() == [[1]]   # [1 | 2^24, 1] with the larger node second


def test_monotone_in_capacity_and_bandwidth_and_exact_scaling():
    rng = np.random.default_rng(3)
    for seed in range(40):
        w = W.random_instances(200 + seed, 1, 12, 4, capacity_factor=1.3)
        t, m, M, B = w.t[0], w.m[0], w.M[0], w.B[0]
        base = O.subset_dp(t, m, M, B)[0][0]
        j = int(rng.integers(4))
        M2 = M.copy(); M2[j] *= np.float32(1.5)
        assert O.subset_dp(t, m, M2, B)[0][0] <= base
        a, b = rng.choice(4, 2, replace=False)
        B2 = B.copy(); B2[a, b] = B2[b, a] = B[a, b] * np.float32(1.7)
        assert O.subset_dp(t, m, M, B2)[0][0] <= base
        for route in ("exhaustive", "subset_dp"):
            b1, c1, o1 = ROUTES[route](t, m, M, B)
            b2, c2, o2 = ROUTES[route](t * np.float32(2), m, M, B)
            if np.isinf(b1[0]):
                assert np.isinf(b2[0])
            else:
                assert bits(b2)[0] == bits(b1 * np.float32(2))[0]      # power-of-two scaling is exact
                assert np.array_equal(c1, c2) and np.array_equal(o1, o2)


def test_relabelling_the_nodes_keeps_beta():
    rng = np.random.default_rng(5)
    for seed in range(40):
        w = W.random_instances(400 + seed, 1, 11, 4, capacity_factor=1.4)
        t, m, M, B = w.t[0], w.m[0], w.M[0], w.B[0]
        p = rng.permutation(4)
        b1, c1, o1, _ = O.exhaustive(t, m, M, B)
        b2, c2, o2, _ = O.exhaustive(t, m, M[p], B[np.ix_(p, p)])
        assert bits(b1)[0] == bits(b2)[0]
        if np.isfinite(b1[0]):
            # the relabelled winner, mapped back, is a feasible solution of the original with the same beta
            back = p[o2[0]]
            beta, ok = O.evaluate(t, m, M, B, back, c2[0])
            assert ok and bits(beta) == bits(b1)[0]


@pytest.mark.parametrize("name,n", [("tiny", 256), ("resnet50_shaped", 64), ("transformer_encoder", 16),
                                    ("headline", 8), ("large", 1)])
def test_certificate_and_lower_bounds_on_the_workloads(name, n):
    """The returned (ordering, cuts) re-evaluated from the definition gives exactly beta and is feasible;
    Theorem 1 (Sec. III-B): beta >= max chosen transfer size / max bandwidth; and beta is at least the
    smallest transfer size over the largest bandwidth."""
    w = W.WORKLOADS[name]().take(n)
    beta, cuts, order = O.subset_dp(w.t, w.m, w.M, w.B)
    assert O.check_inputs(w.t, w.m, w.M, w.B) == 0
    for j in range(w.n_inst):
        if np.isinf(beta[j]):
            assert (order[j] == -1).all() and (cuts[j] == -1).all()
            continue
        assert sorted(order[j].tolist()) == list(range(w.k))
        assert (np.diff(np.concatenate([[0], cuts[j], [w.L]])) > 0).all()
        b, ok = O.evaluate(w.t[j], w.m[j], w.M[j], w.B[j], order[j], cuts[j])
        assert ok and bits(b) == bits(beta)[j]
        bmax = w.B[j].max()
        chosen = w.t[j][cuts[j] - 1]
        assert beta[j] >= chosen.max() / bmax                     # Theorem 1, fp32 quotients are monotone
        assert beta[j] >= w.t[j][: w.L - 1].min() / bmax


def test_exhaustive_matches_subset_dp_on_the_resnet_workload():
    w = W.resnet50_shaped().take(96)
    a = O.exhaustive(w.t, w.m, w.M, w.B)
    b = O.subset_dp(w.t, w.m, w.M, w.B)
    assert np.array_equal(bits(a[0]), bits(b[0])) and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])


def test_transformer_workload_is_dominated_by_ties():
    w = W.transformer_encoder().take(1)
    per, _ = O.eval_orderings(w.t[0], w.m[0], w.M[0], w.B[0], 0, 5040)
    assert len(np.unique(bits(per))) < 100


def test_rank_ranges_compose():
    """The minimum over two halves of the rank range, with the lower rank winning ties, is the whole search."""
    w = W.random_instances(9, 6, 9, 4, quantised=True)
    whole = O.exhaustive(w.t, w.m, w.M, w.B)
    lo = O.exhaustive(w.t, w.m, w.M, w.B, rank_range=(0, 11))
    hi = O.exhaustive(w.t, w.m, w.M, w.B, rank_range=(11, 24))
    for j in range(w.n_inst):
        pick = lo if lo[0][j] <= hi[0][j] else hi
        assert bits(pick[0])[j] == bits(whole[0])[j]
        assert np.array_equal(pick[1][j], whole[1][j]) and np.array_equal(pick[2][j], whole[2][j])


def test_precondition_violations_are_rejected():
    w = W.random_instances(1, 1, 6, 3)
    t, m, M, B = w.t.copy(), w.m.copy(), w.M.copy(), w.B.copy()
    assert O.check_inputs(t, m, M, B) == 0
    B2 = B.copy(); B2[0, 0, 1] *= np.float32(1.5)
    assert O.check_inputs(t, m, M, B2) == -3          # not symmetric
    B3 = B.copy(); B3[0, 1, 2] = B3[0, 2, 1] = 0.0
    assert O.check_inputs(t, m, M, B3) == -3          # zero bandwidth
    t2 = t.copy(); t2[0, 2] = -1.0
    assert O.check_inputs(t2, m, M, B) == -3
    t3 = t.copy(); t3[0, 1] = -0.0
    assert O.check_inputs(t3, m, M, B) == 0           # a zero of either sign is a size of zero
    m2 = m.copy(); m2[0, 0] = np.nan
    assert O.check_inputs(t, m2, M, B) == -3
    with pytest.raises(O.OracleError):
        O.exhaustive(t2, m, M, B)
    # k > L
    assert O.check_inputs(t[:, :2], m[:, :2], M, B) == -1


def test_a_zero_transfer_size_of_either_sign_takes_no_time():
    """Sec. III-B, Eq. 3 with t = 0: nothing is sent, gamma = +0.  A zero that carries a sign bit is still a
    zero: every route gives what it gives for +0, and never the bit pattern of -0."""
    w = W.random_instances(21, 40, 7, 3, capacity_factor=2.0)
    t = w.t.copy()
    t[:, ::2] = np.float32(-0.0)
    plus = np.abs(t)
    assert np.signbit(t).any() and not np.signbit(plus).any()
    for route in (O.bruteforce, lambda *a: O.exhaustive(*a)[:3], O.subset_dp):
        got, ref = route(t, w.m, w.M, w.B), route(plus, w.m, w.M, w.B)
        assert np.array_equal(got[0].view(np.uint32), ref[0].view(np.uint32))
        assert np.array_equal(got[1], ref[1]) and np.array_equal(got[2], ref[2])
        assert not (got[0].view(np.uint32) == 0x80000000).any() and (got[0].view(np.uint32) == 0).any()
    from oracle import ppo_cluster_oracle as CO
    for i in range(6):
        a = CO.bruteforce(t[i], w.m[i], w.M[i], w.B[i])
        b = CO.bruteforce(plus[i], w.m[i], w.M[i], w.B[i])
        assert np.float32(a[0]).view(np.uint32) == np.float32(b[0]).view(np.uint32) != 0x80000000
        assert a[1] == b[1] and np.array_equal(a[2], b[2]) and np.array_equal(a[3], b[3])
