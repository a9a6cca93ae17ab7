"""Pins of the CPU oracle of the search with the compute-time term (oracle/ppo_ct_oracle.c; Sec. I, Eq. 1):
what the paper's definition and plain arithmetic fix, not the oracle against itself."""
import itertools
import math

import numpy as np
import pytest

from oracle import ppo_ct_oracle as CT
from oracle import ppo_oracle as O
from paper_2210_12219_amd import workloads as W


def bits(x):
    return np.asarray(x, dtype=np.float32).view(np.uint32)


ROUTES = {"bruteforce": CT.bruteforce, "exhaustive": CT.exhaustive, "subset_dp": CT.subset_dp}


@pytest.mark.parametrize("route", ROUTES)
def test_without_work_the_term_vanishes(route):
    """w = 0: every compute stage is +0 and Eq. 1 reduces to Eq. 2, whose oracle is pinned on its own."""
    f = ROUTES[route]
    for seed, (L, k) in enumerate([(7, 3), (9, 4), (6, 2), (5, 5), (8, 1)]):
        w = W.random_instances(600 + seed, 12, L, k, capacity_factor=1.5, quantised=bool(seed % 2))
        ref = O.bruteforce(w.t, w.m, w.M, w.B)
        rng = np.random.default_rng(seed)
        for i in range(w.n_inst):
            v = rng.uniform(0.5, 3.0, k).astype(np.float32)
            b, cuts, order = f(w.t[i], w.m[i], np.zeros(L, np.float32), w.M[i], v, w.B[i])
            assert bits(b) == bits(ref[0][i]), (route, seed, i)
            assert np.array_equal(cuts, ref[1][i]) and np.array_equal(order, ref[2][i])


@pytest.mark.parametrize("route", ROUTES)
def test_one_node_is_the_whole_work_over_its_speed(route):
    """k = 1: beta = (sum of the work) / v, summed in binary64 and rounded once; +inf if the model does not fit."""
    f = ROUTES[route]
    work = np.array([0.1, 0.2, 0.3, 0.7, 1.1], np.float32)
    total = 0.0
    for x in work:
        total += float(x)
    v = np.float32(3.0)
    b, cuts, order = f(np.ones(5, np.float32), np.ones(5, np.float32), work, np.array([5.0], np.float32),
                       np.array([v]), np.zeros((1, 1), np.float32))
    assert bits(b) == bits(np.float32(total / float(v))) and list(order) == [0]
    b, _, order = f(np.ones(5, np.float32), np.ones(5, np.float32), work, np.array([4.5], np.float32),
                    np.array([v]), np.zeros((1, 1), np.float32))
    assert np.isinf(b) and list(order) == [-1]


@pytest.mark.parametrize("route", ROUTES)
def test_equal_work_no_transfers_no_memory_limit(route):
    """t = 0, unit work, equal speeds v, ample memory: the best cut into k non-empty segments has a longest
    segment of ceil(L / k) layers, so beta = ceil(L / k) / v; the identity ordering wins the tie; the cut rule
    (last cut as small as possible, then the one before, ...) puts the long segments last."""
    f = ROUTES[route]
    for L, k, v in ((7, 3, 2.0), (8, 4, 1.0), (9, 2, 4.0), (5, 5, 0.5)):
        b, cuts, order = f(np.zeros(L, np.float32), np.ones(L, np.float32), np.ones(L, np.float32),
                           np.full(k, 100.0, np.float32), np.full(k, v, np.float32),
                           np.ones((k, k), np.float32) - np.eye(k, dtype=np.float32))
        longest = math.ceil(L / k)
        assert float(b) == longest / v and list(order) == list(range(k))
        want, e = [], L
        for s in range(k - 1, 0, -1):          # segment s takes as many layers as the bound and the rest allow
            e = max(e - longest, s)
            want.append(e)
        assert list(cuts) == want[::-1]


@pytest.mark.parametrize("route", ROUTES)
def test_a_slow_node_gets_the_light_end(route):
    """Worked by hand.  Work 8, 1, 1 on nodes of speed 8 and 1, no transfers, no memory limit.  Two segments:
    cut after layer 1: fast node first 8/8 = 1 and 2/1 = 2 -> 2; slow node first 8/1 = 8.  Cut after layer 2:
    fast first 9/8 and 1/1 -> 1.125; slow first 9 and 1/8 -> 9.  Optimum 1.125: order (0, 1), cut 2."""
    f = ROUTES[route]
    b, cuts, order = f(np.zeros(3, np.float32), np.ones(3, np.float32), np.array([8, 1, 1], np.float32),
                       np.full(2, 10.0, np.float32), np.array([8, 1], np.float32),
                       np.array([[0, 1], [1, 0]], np.float32))
    assert float(b) == 1.125 and list(cuts) == [2] and list(order) == [0, 1]
    # the same with a transfer that costs more than it saves: t = (0, 5) over a link of 2 -> cut 2 costs 2.5,
    # cut 1 costs max(0, 2) = 2: optimum 2 at cut 1
    b, cuts, order = f(np.array([0, 5, 0], np.float32), np.ones(3, np.float32), np.array([8, 1, 1], np.float32),
                       np.full(2, 10.0, np.float32), np.array([8, 1], np.float32),
                       np.array([[0, 2], [2, 0]], np.float32))
    assert float(b) == 2.0 and list(cuts) == [1] and list(order) == [0, 1]


@pytest.mark.parametrize("route", ROUTES)
def test_compute_stage_is_divided_in_binary64_and_rounded_once(route):
    """Work 23642438 + 41 on a node of speed 56, one segment: the sum 23642479 is exact in binary64 but not in
    binary32 (it would round to 23642480); 23642479 / 56 = 422187.125 exactly, so beta = 422187.125, while a
    binary32 sum or quotient gives 422187.15625 (by hand: 23642480 / 56 = 422187.1428..., nearest float above .125)."""
    f = ROUTES[route]
    b, cuts, order = f(np.zeros(2, np.float32), np.ones(2, np.float32), np.array([23642438, 41], np.float32),
                       np.array([5.0], np.float32), np.array([56.0], np.float32), np.zeros((1, 1), np.float32))
    assert float(b) == 422187.125


def definition(t, m, w, M, v, B):
    """Eq. 1 written out in Python (binary64 sums, one rounding), every (permutation, cut vector) pair."""
    L, k = len(t), len(M)
    P = np.concatenate([[0.0], np.cumsum(m.astype(np.float64))])
    Q = [0.0]
    for x in w:
        Q.append(Q[-1] + float(x))
    best = None
    for rank, perm in enumerate(itertools.permutations(range(k))):
        for cuts in itertools.combinations(range(1, L), k - 1):
            c = (0,) + cuts + (L,)
            if any(P[c[s + 1]] - P[c[s]] > float(M[perm[s]]) for s in range(k)):
                continue
            stages = [np.float32((Q[c[s + 1]] - Q[c[s]]) / float(v[perm[s]])) for s in range(k)]
            stages += [np.float32(t[c[s] - 1]) / np.float32(B[perm[s - 1], perm[s]]) for s in range(1, k)]
            b = max(stages)
            key = (b, rank, tuple(reversed(cuts)))
            if best is None or key < best[0]:
                best = (key, perm, cuts)
    if best is None:
        return np.float32(np.inf), [-1] * (k - 1), [-1] * k
    return np.float32(best[0][0]), list(best[2]), list(best[1])


def test_the_three_routes_against_the_definition_written_out():
    rng = np.random.default_rng(5)
    n_inf = 0
    for seed in range(60):
        L = int(rng.integers(2, 8))
        k = int(rng.integers(1, min(L, 4) + 1))
        w = W.random_instances(700 + seed, 1, L, k, capacity_factor=float(rng.uniform(1.0, 2.0)), quantised=bool(seed % 2))
        work, speed = W.compute_terms(w, seed=seed, seconds=float(rng.uniform(0.2, 5.0)), quantised=bool(seed % 3 == 0))
        ref = definition(w.t[0], w.m[0], work[0], w.M[0], speed[0], w.B[0])
        n_inf += bool(np.isinf(ref[0]))
        for name, f in ROUTES.items():
            b, cuts, order = f(w.t[0], w.m[0], work[0], w.M[0], speed[0], w.B[0])
            assert bits(b) == bits(ref[0]), (seed, name, b, ref[0])
            assert list(cuts) == ref[1] and list(order) == ref[2], (seed, name)
    assert 3 <= n_inf <= 40


def test_routes_agree_at_larger_sizes_and_the_solution_evaluates_to_beta():
    for seed, (L, k) in enumerate([(14, 5), (20, 6), (30, 5), (12, 7)]):
        w = W.random_instances(800 + seed, 3, L, k, capacity_factor=1.4, quantised=bool(seed % 2))
        work, speed = W.compute_terms(w, seed=seed, seconds=2.0, quantised=bool(seed % 2))
        for i in range(w.n_inst):
            a = CT.exhaustive(w.t[i], w.m[i], work[i], w.M[i], speed[i], w.B[i])
            b = CT.subset_dp(w.t[i], w.m[i], work[i], w.M[i], speed[i], w.B[i])
            assert bits(a[0]) == bits(b[0]) and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
            if np.isfinite(a[0]):
                beta, feas = CT.evaluate(w.t[i], w.m[i], work[i], w.M[i], speed[i], w.B[i], a[2], a[1])
                assert feas and bits(beta) == bits(a[0])
            per = CT.eval_orderings(w.t[i], w.m[i], work[i], w.M[i], speed[i], w.B[i], 0, math.factorial(k))
            assert bits(per.min()) == bits(a[0])
            if np.isfinite(a[0]):
                assert int(np.argmin(per)) == O.rank(a[2])


def test_invariants():
    """More work never helps; beta is at least the optimum without the term and at least the lightest possible
    heaviest stage; doubling the work and halving nothing else doubles pure compute optima exactly."""
    w = W.random_instances(900, 10, 10, 4, capacity_factor=1.6)
    work, speed = W.compute_terms(w, seed=1, seconds=3.0)
    base = O.bruteforce(w.t, w.m, w.M, w.B)
    for i in range(w.n_inst):
        b1 = CT.subset_dp(w.t[i], w.m[i], work[i], w.M[i], speed[i], w.B[i])[0]
        b2 = CT.subset_dp(w.t[i], w.m[i], work[i] * np.float32(2), w.M[i], speed[i], w.B[i])[0]
        b3 = CT.subset_dp(w.t[i], w.m[i], work[i], w.M[i], speed[i] * np.float32(2), w.B[i])[0]
        assert bits(base[0][i]) <= bits(b3) <= bits(b1) <= bits(b2)
        if np.isfinite(b1):
            assert float(b1) >= float(work[i].max()) / float(speed[i].max()) * (1 - 1e-6)
        z = np.zeros_like(w.t[i])
        p1 = CT.subset_dp(z, w.m[i], work[i], w.M[i], speed[i], w.B[i])[0]
        p2 = CT.subset_dp(z, w.m[i], work[i] * np.float32(2), w.M[i], speed[i], w.B[i])[0]
        assert bits(p2) == bits(np.float32(2) * p1)


def test_bad_inputs_are_refused():
    w = W.random_instances(1, 1, 6, 3)
    work, speed = W.compute_terms(w)
    args = [w.t[0], w.m[0], work[0], w.M[0], speed[0], w.B[0]]
    bad_speed = speed[0].copy(); bad_speed[1] = 0
    bad_work = work[0].copy(); bad_work[2] = -1
    for a in ([*args[:4], bad_speed, args[5]], [*args[:2], bad_work, *args[3:]]):
        with pytest.raises(CT.OracleError):
            CT.bruteforce(*a)
