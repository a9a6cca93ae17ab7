"""Random small problems through every route of the library, each against the CPU oracles, bit for bit.

The shapes are drawn per seed: k, L and the batch size for the fixed-k routes (enumeration, shared prefix with
a bound, subset DP), the cluster size, the segment limit and the capacity regime for the cluster form, a random
capacity per instance for the partitioning step.  The named workloads fix their shapes; this file moves them."""
import math

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import ppo_cluster_oracle as CO
from oracle import ppo_oracle as O
from oracle import ppo_partition_oracle as PO
from paper_2210_12219_amd import workloads as W

SEEDS = range(1, 401)


@pytest.fixture(scope="module")
def ppo():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2210_12219_amd import binding
    binding.load()
    return binding


def bits(x):
    return np.asarray(x, dtype=np.float32).view(np.uint32)


def same(got, ref, what):
    assert np.array_equal(bits(got[0]), bits(ref[0])), what + ": beta"
    assert np.array_equal(got[2], ref[2]), what + ": ordering"
    assert np.array_equal(got[1], ref[1]), what + ": cuts"


def test_fixed_k_routes_on_random_shapes(ppo):
    import torch
    for seed in SEEDS:
        rng = np.random.default_rng(410000 + seed)
        k = int(rng.integers(1, 10))
        L = int(rng.integers(k, min(128, k + 60) + 1))
        if k >= 8:
            L = min(L, k + 30)
        n_inst = int(rng.integers(1, 6)) if k >= 8 else int(rng.integers(1, 20))
        w = W.random_instances(410000 + seed, n_inst, L, k, capacity_factor=float(rng.uniform(1.0, 2.0)),
                               quantised=bool(seed % 2))
        what = f"seed {seed} k={k} L={L} n_inst={n_inst}"
        ref = O.subset_dp(w.t, w.m, w.M, w.B)
        dev = ppo.to_device(w)
        got = tuple(x.cpu().numpy() for x in ppo.ppo_solve(*dev))
        same(got, ref, what + " enumeration")
        ws = ppo.alloc_workspace(L, k, n_inst)
        for route in ("bounded", "subsets"):
            keys = torch.empty(n_inst, dtype=torch.int64, device="cuda:0")
            ppo.ppo_prepare(*dev, ws)
            ppo.ppo_init_keys(keys)
            if route == "bounded":
                ppo.ppo_solve_range_bounded(L, k, n_inst, ws, 0, math.factorial(k), keys, None)
            else:
                ppo.ppo_solve_subsets(L, k, n_inst, ws, keys)
            out = tuple(x.cpu().numpy() for x in ppo.ppo_finalize(L, k, n_inst, ws, keys))
            torch.cuda.synchronize()
            same(out, ref, what + " " + route)


def test_cluster_and_partition_on_random_shapes(ppo):
    import torch
    for seed in SEEDS:
        rng = np.random.default_rng(420000 + seed)
        n = int(rng.integers(1, 13))
        L = int(rng.integers(1, 129))
        if n >= 10:
            L = min(L, 60)
        pmax = int(rng.integers(1, n + 1))
        n_inst = int(rng.integers(1, 5))
        # two capacity regimes: nodes that hold a good part of the model each, and nodes that hold about 1/n
        cf = float(rng.uniform(0.3, 1.2) * n) if seed % 3 else float(rng.uniform(0.8, 1.5))
        w = W.random_instances(420000 + seed, n_inst, L, n, capacity_factor=cf, quantised=bool((seed // 2) % 2))
        what = f"seed {seed} n={n} L={L} pmax={pmax} n_inst={n_inst}"
        out = tuple(x.cpu().numpy() for x in ppo.ppo_solve_cluster(*ppo.to_device(w), max_segments=pmax))
        torch.cuda.synchronize()
        for i in range(n_inst):
            beta, p, cuts, order = CO.subset_dp(w.t[i], w.m[i], w.M[i], w.B[i], pmax)
            assert bits(out[0][i]) == bits(beta) and out[1][i] == p, f"{what} instance {i}: beta or segment count"
            assert np.array_equal(out[2][i], cuts) and np.array_equal(out[3][i], order), f"{what} instance {i}: cuts or nodes"
        kappa = rng.uniform(0.5, 3.0, n_inst).astype(np.float32) * np.float32(w.m.sum() / n_inst / max(1, n))
        dev = [torch.tensor(np.ascontiguousarray(x, dtype=np.float32), device="cuda:0") for x in (w.t, w.m, kappa)]
        segs, cuts, total = (x.cpu().numpy() for x in ppo.ppo_min_sum_partition(*dev))
        torch.cuda.synchronize()
        for i in range(n_inst):
            p, c, s = PO.partition(w.t[i], w.m[i], kappa[i])
            assert segs[i] == p and list(cuts[i][:max(p - 1, 0)]) == list(c), f"{what} instance {i}: partition"
            assert total[i] == s or (np.isinf(total[i]) and np.isinf(s)), f"{what} instance {i}: partition sum"
