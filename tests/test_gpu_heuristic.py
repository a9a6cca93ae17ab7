"""The paper's placement algorithm and its comparison systems on the GPU (ppo_place_kpath, ppo_place_baseline)
against their oracle, element by element; and the comparison the exact search makes possible."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import ppo_heuristic_oracle as H
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


def run_kpath(ppo, w, kappa, n_classes):
    import torch
    t, m, _, B = ppo.to_device(w)
    out = ppo.ppo_place_kpath(t, m, torch.from_numpy(np.ascontiguousarray(kappa, np.float32)).cuda(), B, n_classes)
    torch.cuda.synchronize()
    return tuple(x.cpu().numpy() for x in out)


def check_kpath(ppo, w, kappa, n_classes, what):
    beta, segs, cuts, order, used = run_kpath(ppo, w, kappa, n_classes)
    for i in range(w.n_inst):
        rb, rp, rcuts, rnodes, rused = H.heuristic(w.t[i], w.m[i], kappa[i], w.B[i], n_classes)
        assert bits(beta[i]) == bits(rb) and segs[i] == rp and used[i] == rused, (what, i, beta[i], rb, segs[i], rp, used[i], rused)
        assert list(cuts[i][:max(rp - 1, 0)]) == list(rcuts) and (cuts[i][max(rp - 1, 0):] == -1).all(), (what, i)
        assert list(order[i][:rp]) == list(rnodes) and (order[i][rp:] == -1).all(), (what, i, order[i], rnodes)
    return beta, segs


def test_paper_shaped_clusters(ppo):
    """Sec. IV: 5 to 50 devices of one capacity, Shannon-rate bandwidths, 2 to 20 classes."""
    for n, cap in ((5, 32), (10, 32), (10, 16), (15, 24), (20, 16), (50, 16), (50, 64)):
        w = W.cluster_geometric(n, cap, n_inst=6, seed=60 + n)
        for nc in (2, 5, 20):
            print(f"heuristic geometric n={n} cap={cap} classes={nc}", flush=True)
            beta, segs = check_kpath(ppo, w, w.M[:, 0].copy(), nc, f"geometric n={n} cap={cap} nc={nc}")
            assert np.isfinite(beta).all() and (segs >= 2).all()


def test_mixed_bandwidths_many_partitions(ppo):
    """Log-uniform bandwidths (every link different) and a capacity that needs many partitions."""
    for n, frac, L in ((8, 0.25, 100), (12, 0.12, 100), (20, 0.08, 128), (30, 0.05, 100)):
        w = W.cluster_mixed(n, L=L, n_inst=4, seed=70 + n)
        kappa = (frac * w.m.sum(axis=1)).astype(np.float32)
        for nc in (1, 3, 8):
            print(f"heuristic mixed n={n} L={L} classes={nc}", flush=True)
            check_kpath(ppo, w, kappa, nc, f"mixed n={n} nc={nc}")


def test_small_shapes_and_failures(ppo):
    for seed in range(25):
        rng = np.random.default_rng(9100 + seed)
        L, n = int(rng.integers(1, 14)), int(rng.integers(1, 9))
        w = W.random_instances(seed, 12, L, n, capacity_factor=1.0, quantised=bool(seed % 2))
        kappa = (w.m.sum(axis=1) * rng.uniform(0.15, 1.1, w.n_inst)).astype(np.float32)
        print(f"heuristic small seed={seed} L={L} n={n}", flush=True)
        beta, segs = check_kpath(ppo, w, kappa, int(rng.integers(1, 6)), f"small seed={seed}")
    # more partitions than nodes, and a layer that fits no node
    w = W.random_instances(1, 4, 10, 3, capacity_factor=1.0)
    beta, segs = check_kpath(ppo, w, (1.01 * w.m.max(axis=1)).astype(np.float32), 3, "too many partitions")
    assert np.isinf(beta).any()
    beta, segs = check_kpath(ppo, w, np.full(4, 0.5 * float(w.m.min()), np.float32), 3, "nothing fits")
    assert np.isinf(beta).all() and (segs == 0).all()


def test_search_budget_is_the_same_on_both_sides(ppo):
    """Two groups of 12 nodes with fast links inside and slow ones between, 14 partitions in one class: at the
    thresholds that cut the groups apart no path of 14 nodes exists, and finding that out by depth-first search
    takes more than the budget, so both sides give up there in the same way."""
    n, L = 24, 28
    rng = np.random.default_rng(5)
    B = np.zeros((n, n), np.float32)
    for a in range(n):
        for b in range(a + 1, n):
            B[a, b] = B[b, a] = (rng.uniform(50, 100) if (a < 12) == (b < 12) else rng.uniform(1, 2))
    t = rng.uniform(1, 9, (1, L)).astype(np.float32)
    m = np.ones((1, L), np.float32)
    w = W.Workload("two groups", L, n, 1, 5, t, m, np.full((1, n), 2.0, np.float32), B[None])
    beta, segs = check_kpath(ppo, w, np.array([2.0], np.float32), 1, "two groups")
    assert segs[0] >= 14 and np.isfinite(beta[0])


def test_comparison_systems(ppo):
    import torch
    for n, cap, seed in ((5, 32, 1), (10, 16, 2), (20, 16, 3), (50, 24, 4)):
        w = W.cluster_geometric(n, cap, n_inst=8, seed=80 + seed)
        t, m, _, B = ppo.to_device(w)
        kappa = torch.from_numpy(np.ascontiguousarray(w.M[:, 0])).cuda()
        print(f"comparison systems n={n} cap={cap}", flush=True)
        jb, js, jc, jo = (x.cpu().numpy() for x in ppo.ppo_place_baseline(t, m, kappa, B, ppo.PPO_BASELINE_JOINT))
        draws = np.random.default_rng(seed).random((w.n_inst, 40)).astype(np.float32)
        rb, rs, rc, ro = (x.cpu().numpy() for x in ppo.ppo_place_baseline(t, m, kappa, B, ppo.PPO_BASELINE_RANDOM,
                                                                        torch.from_numpy(draws).cuda()))
        torch.cuda.synchronize()
        for i in range(w.n_inst):
            for got, ref in (((jb, js, jc, jo), H.joint_baseline(w.t[i], w.m[i], w.M[i][0], w.B[i])),
                             ((rb, rs, rc, ro), H.random_baseline(w.t[i], w.m[i], w.M[i][0], w.B[i], draws[i]))):
                b, p, cuts, nodes = ref
                assert bits(got[0][i]) == bits(b) and got[1][i] == p, (n, i, got[0][i], b)
                if p:
                    assert list(got[2][i][:p - 1]) == list(cuts) and list(got[3][i][:p]) == list(nodes)


def test_the_exact_optimum_is_never_beaten(ppo):
    """Sec. V's approximation ratio with the true optimum in place of Theorem 1's bound."""
    import torch
    for n, cap in ((5, 32), (10, 32), (15, 24)):
        w = W.cluster_geometric(n, cap, n_inst=16, seed=90 + n)
        exact = ppo.ppo_solve_cluster(*ppo.to_device(w))[0].cpu().numpy()
        heur = run_kpath(ppo, w, w.M[:, 0].copy(), 5)[0]
        torch.cuda.synchronize()
        assert (bits(exact) <= bits(heur)).all() and np.isfinite(heur).all()
