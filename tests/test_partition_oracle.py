"""Pins for the oracle of the paper's partitioning step (oracle/ppo_partition_oracle.py)."""
import math

import numpy as np

from oracle import ppo_partition_oracle as PO


def test_closed_forms():
    t = [5.0, 1.0, 7.0, 2.0, 9.0]
    m = [2.0, 2.0, 2.0, 2.0, 2.0]
    for f in (PO.bruteforce, PO.partition):
        assert f(t, m, 10.0) == (1, (), 0.0)                               # everything fits one node
        assert f(t, m, 2.0) == (5, (1, 2, 3, 4), 5.0 + 1.0 + 7.0 + 2.0)    # one layer per node: every cut is paid
        assert f(t, m, 1.0) == (0, (), math.inf)                           # a layer that fits nowhere
        # capacity 6 = three layers: two segments are enough, the cut after layer 2 (t = 1) or 3 (t = 7): the cheaper
        assert f(t, m, 6.0) == (2, (2,), 1.0)
        # capacity 4 = two layers: at least three segments; cuts {2, 4}: 1 + 2 = 3 beats {1, 3}: 5 + 7 and {2, 3}..
        assert f(t, m, 4.0) == (3, (2, 4), 3.0)
    # ties: equal sums -> fewest segments, then the smallest cuts
    t2 = [1.0, 1.0, 1.0, 0.0]
    m2 = [1.0, 1.0, 1.0, 1.0]
    for f in (PO.bruteforce, PO.partition):
        assert f(t2, m2, 2.0) == (2, (2,), 1.0)
        assert f([0.0, 0.0, 0.0, 0.0], m2, 3.0) == (2, (1,), 0.0)


def test_routes_agree_on_integer_instances():
    rng = np.random.default_rng(1)
    for _ in range(300):
        L = int(rng.integers(1, 11))
        t = rng.integers(0, 6, L).astype(float)
        m = rng.integers(1, 7, L).astype(float)
        kappa = float(rng.integers(3, 16))
        assert PO.bruteforce(t, m, kappa) == PO.partition(t, m, kappa)


def test_sums_agree_on_real_valued_instances():
    """Rounded addition is monotone, so the least sum is the same by both routes even when sums round; the cuts
    returned always reproduce it."""
    rng = np.random.default_rng(2)
    for _ in range(200):
        L = int(rng.integers(2, 11))
        t = rng.uniform(0.1, 30.0, L).astype(np.float32)
        m = rng.uniform(0.1, 50.0, L).astype(np.float32)
        kappa = float(np.float32(rng.uniform(40.0, 150.0)))
        pa, ca, sa = PO.bruteforce(t, m, kappa)
        pb, cb, sb = PO.partition(t, m, kappa)
        assert sa == sb and (pa == 0) == (pb == 0)
        if pb:
            total = 0.0
            for c in reversed(cb):
                total = float(t[c - 1]) + total
            assert total == sb and len(cb) == pb - 1


def test_order_of_addition_is_immaterial_on_the_tested_inputs():
    """The definition fixes an order of addition (from the chain's end) only so that the sum is defined when it
    rounds.  The sizes used in the tests and workloads are binary32 values within a few binary orders of one
    another: sums of up to 128 of them are exact in binary64, so any order gives the same bits.  Checked here
    against the correctly rounded sum (math.fsum), for every set of cuts of the brute-force route."""
    import itertools
    rng = np.random.default_rng(3)
    for _ in range(100):
        L = int(rng.integers(2, 11))
        t = rng.uniform(0.1, 30.0, L).astype(np.float32)
        for p in range(1, L + 1):
            for cuts in itertools.combinations(range(1, L), p - 1):
                ordered = 0.0
                for c in reversed(cuts):
                    ordered = float(t[c - 1]) + ordered
                forward = 0.0
                for c in cuts:
                    forward = forward + float(t[c - 1])
                assert ordered == forward == math.fsum(float(t[c - 1]) for c in cuts)
    # and at the sizes the GPU tests use: 128 sizes spanning three decimal orders
    t = np.exp(rng.uniform(np.log(0.05), np.log(60.0), 128)).astype(np.float32)
    back = 0.0
    for x in t[::-1]:
        back = float(x) + back
    assert back == math.fsum(float(x) for x in t) == float(np.sum(t.astype(np.float64)))
