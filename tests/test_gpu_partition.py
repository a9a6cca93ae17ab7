"""The paper's partitioning step on the GPU (ppo_min_sum_partition) against its oracle, and what it costs to
partition first and place afterwards instead of searching jointly."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import ppo_cluster_oracle as CO
from oracle import ppo_partition_oracle as PO
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


def run(ppo, t, m, kappa):
    import torch
    dev = [torch.tensor(np.ascontiguousarray(x, dtype=np.float32), device="cuda:0") for x in (t, m, kappa)]
    segs, cuts, total = ppo.ppo_min_sum_partition(*dev)
    torch.cuda.synchronize()
    return segs.cpu().numpy(), cuts.cpu().numpy(), total.cpu().numpy()


def test_partition_matches_the_oracle(ppo):
    rng = np.random.default_rng(4)
    for case in range(60):
        L = int(rng.integers(1, 129)) if case % 4 else int(rng.integers(1, 8))
        n = int(rng.integers(1, 40))
        if case % 2:
            t = rng.integers(0, 6, (n, L)).astype(np.float32)
            m = rng.integers(1, 7, (n, L)).astype(np.float32)
            kappa = rng.integers(3, 40, n).astype(np.float32)
        else:
            t = rng.uniform(0.1, 30.0, (n, L)).astype(np.float32)
            m = rng.uniform(0.1, 50.0, (n, L)).astype(np.float32)
            kappa = rng.uniform(30.0, 400.0, n).astype(np.float32)
        print(f"partition case {case} L={L} n={n}", flush=True)
        segs, cuts, total = run(ppo, t, m, kappa)
        for i in range(n):
            p, c, s = PO.partition(t[i], m[i], kappa[i])
            assert segs[i] == p and (total[i] == s or (np.isinf(total[i]) and np.isinf(s))), (case, i)
            assert list(cuts[i][:max(p - 1, 0)]) == list(c) and list(cuts[i][max(p - 1, 0):]) == [-1] * (L - 1 - max(p - 1, 0))


@pytest.mark.parametrize("n,cap", [(5, 32), (10, 32), (10, 48), (15, 24)])
def test_partition_then_place_against_the_joint_optimum(ppo, n, cap):
    """Sec. III-B: the paper partitions first (least sum of transfer sizes) and places afterwards.  For that fixed
    partition the best placement is what the cluster search finds on the chain of merged segments; it cannot
    beat the joint optimum, and Theorem 1's bound max(S) / max(B) cannot beat it."""
    import torch
    w = W.cluster_geometric(n, cap, n_inst=6, seed=21)
    kappa = np.full(w.n_inst, cap, np.float32)
    segs, cuts, total = run(ppo, w.t, w.m, kappa)
    joint = tuple(x.cpu().numpy() for x in ppo.ppo_solve_cluster(*ppo.to_device(w)))
    torch.cuda.synchronize()
    print(f"partition then place n={n} capacity={cap}", flush=True)
    worse = 0
    for i in range(w.n_inst):
        p = int(segs[i])
        assert (p == 0) == np.isinf(joint[0][i]) or p > n     # the partition ignores how many nodes there are
        if p == 0 or p > n:
            continue
        c = [0] + [int(x) for x in cuts[i][:p - 1]] + [w.L]
        m2 = np.array([w.m[i][a:b].astype(np.float64).sum() for a, b in zip(c[:-1], c[1:])], np.float32)
        t2 = np.array([w.t[i][b - 1] for b in c[1:]], np.float32)
        # merged segments fit with a little slack for the rounding of their sums to binary32
        M2 = np.full(n, np.float32(cap) * np.float32(1.0001), np.float32)
        dev = [torch.tensor(x[None], device="cuda:0") for x in (t2, m2, M2)] + [torch.tensor(w.B[i][None], device="cuda:0")]
        placed = tuple(x.cpu().numpy() for x in ppo.ppo_solve_cluster(*dev, max_segments=p))
        torch.cuda.synchronize()
        ref = CO.subset_dp(t2, m2, M2, w.B[i], p)
        assert bits(placed[0][0]) == bits(ref[0]) and placed[1][0] == ref[1] == p
        assert bits(joint[0][i]) <= bits(placed[0][0])                       # joint search is never worse
        bound = np.float32(t2[:-1].max()) / np.float32(w.B[i].max())          # Theorem 1 for this partition
        assert bits(bound) <= bits(placed[0][0])
        worse += bits(joint[0][i]) < bits(placed[0][0])
    print(f"   joint optimum strictly better in {worse} of {w.n_inst}", flush=True)
