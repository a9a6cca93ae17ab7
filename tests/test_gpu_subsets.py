"""Stage 2 by dynamic programming over node subsets (ppo_solve_subsets): the same keys as the enumeration of
all orderings, hence the same beta, cuts and ordering as the CPU oracle, bit for bit."""
import math

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import ppo_oracle as O
from paper_2210_12219_amd import workloads as W


@pytest.fixture(scope="module")
def ppo():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2210_12219_amd import binding
    binding.load()
    return binding


def bits(x):
    return np.asarray(x, dtype=np.float32).view(np.uint32)


def solve(ppo, w, route):
    import torch
    dev = ppo.to_device(w)
    ws = ppo.alloc_workspace(w.L, w.k, w.n_inst)
    keys = torch.empty(w.n_inst, dtype=torch.int64, device="cuda:0")
    ppo.ppo_prepare(*dev, ws)
    ppo.ppo_init_keys(keys)
    if route == "subsets":
        ppo.ppo_solve_subsets(w.L, w.k, w.n_inst, ws, keys)
    else:
        ppo.ppo_solve_range(w.L, w.k, w.n_inst, ws, 0, math.factorial(w.k), keys)
    out = ppo.ppo_finalize(w.L, w.k, w.n_inst, ws, keys)
    torch.cuda.synchronize()
    return tuple(x.cpu().numpy() for x in out), keys.cpu().numpy()


def assert_same(got, ref, what=""):
    bad = np.nonzero(bits(got[0]) != bits(ref[0]))[0]
    assert bad.size == 0, f"{what}: beta differs at instances {bad[:8]}: {got[0][bad[:4]]} vs {ref[0][bad[:4]]}"
    assert np.array_equal(got[2], ref[2]), f"{what}: ordering differs"
    assert np.array_equal(got[1], ref[1]), f"{what}: cuts differ"


def same_keys(a, b):
    """keys agree; for infeasible instances (beta = +inf) only the beta half is defined"""
    inf = (a >> 32) == 0x7F800000
    return np.array_equal(a >> 32, b >> 32) and np.array_equal(a[~inf], b[~inf])


def test_subsets_named_workloads(ppo):
    for w in (W.tiny(), W.resnet50_shaped(), W.transformer_encoder(), W.headline(), W.large()):
        got, keys = solve(ppo, w, "subsets")
        ref = O.bruteforce(w.t, w.m, w.M, w.B) if w.k <= 4 else O.subset_dp(w.t, w.m, w.M, w.B)
        assert_same(got, ref, f"{w.name}, subsets route")
        if w.k <= 10:
            assert same_keys(keys, solve(ppo, w, "range")[1]), w.name


def test_subsets_small_shapes_ties_and_infeasible(ppo):
    for seed in range(30):
        rng = np.random.default_rng(6000 + seed)
        L = int(rng.integers(1, 13))
        k = int(rng.integers(1, min(L, 6) + 1))
        w = W.random_instances(seed, 40, L, k, capacity_factor=float(rng.uniform(1.0, 1.8)), quantised=bool(seed % 2))
        ref = O.exhaustive(w.t, w.m, w.M, w.B)[:3] if k >= 5 else O.bruteforce(w.t, w.m, w.M, w.B)
        got, keys = solve(ppo, w, "subsets")
        assert_same(got, ref, f"subsets L={L} k={k} seed={seed}")
        assert same_keys(keys, solve(ppo, w, "range")[1]), (L, k, seed)


def test_subsets_maximum_sizes(ppo):
    """k = 12, L = 128: the enumeration would take 479 million DPs per instance; the oracle's own subset DP
    is the reference."""
    w = W.random_instances(77, 4, 128, 12, capacity_factor=1.3, quantised=False)
    got, _ = solve(ppo, w, "subsets")
    assert_same(got, O.subset_dp(w.t, w.m, w.M, w.B), "subsets at k=12, L=128")
