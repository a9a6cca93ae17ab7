"""Cluster form for large clusters and few segments (ppo_solve_cluster_few; Sec. IV of the paper: 5 to 50 devices):
bit for bit against the CPU oracle of the cluster form where the oracle can go, against ppo_solve_cluster where both
apply, and at the paper's 50 devices through clusters whose answer the oracle can produce."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import ppo_cluster_oracle as CO
from paper_2210_12219_amd import workloads as W
from paper_2210_12219_amd.workloads import Workload


@pytest.fixture(scope="module")
def ppo():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2210_12219_amd import binding
    binding.load()
    return binding


def bits(x):
    return np.asarray(x, dtype=np.float32).view(np.uint32)


def solve_few(ppo, w, pmax, workspace_bytes=None):
    import torch
    dev = ppo.to_device(w)
    ws = None
    if workspace_bytes is not None:
        ws = torch.empty(workspace_bytes, dtype=torch.uint8, device="cuda:0")
    out = ppo.ppo_solve_cluster_few(*dev, max_segments=pmax, workspace=ws)
    torch.cuda.synchronize()
    return tuple(x.cpu().numpy() for x in out)


def oracle(w, pmax, route):
    n = w.k
    beta = np.zeros(w.n_inst, np.float32)
    segs = np.zeros(w.n_inst, np.int32)
    cuts = np.zeros((w.n_inst, max(n - 1, 0)), np.int32)
    order = np.zeros((w.n_inst, n), np.int32)
    for i in range(w.n_inst):
        beta[i], segs[i], cuts[i], order[i] = route(w.t[i], w.m[i], w.M[i], w.B[i], pmax)
    return beta, segs, cuts, order


def assert_same(got, ref, what):
    bad = np.nonzero(bits(got[0]) != bits(ref[0]))[0]
    assert bad.size == 0, f"{what}: beta differs at instances {bad[:8]}: {got[0][bad[:4]]} vs {ref[0][bad[:4]]}"
    assert np.array_equal(got[1], ref[1]), f"{what}: number of segments differs"
    assert np.array_equal(got[3], ref[3]), f"{what}: node sequence differs"
    assert np.array_equal(got[2], ref[2]), f"{what}: cuts differ"


def with_decoys(w, n, rng):
    """the instances of w in clusters of n nodes: the old nodes keep their order among nodes too small for any layer
    (every layer is made to weigh something); returns the workload and, per instance, where the old nodes sit"""
    n0 = w.k
    m = (w.m + np.float32(0.01)).astype(np.float32)
    M = np.zeros((w.n_inst, n), np.float32)
    B = np.zeros((w.n_inst, n, n), np.float32)
    places = []
    for i in range(w.n_inst):
        place = np.sort(rng.permutation(n)[:n0])
        b = rng.uniform(1.0, 100.0, size=(n, n)).astype(np.float32)
        b = np.maximum(b, b.T)
        np.fill_diagonal(b, 0)
        b[np.ix_(place, place)] = w.B[i]
        M[i, place] = w.M[i]
        B[i] = b
        places.append(place)
    return Workload(w.name + f"+decoys{n}", w.L, n, w.n_inst, w.seed, w.t, m, M, B), places


def test_small_shapes_ties_and_infeasible(ppo):
    """Random shapes from n = 1 and L = 1 up, every max_segments, values with few distinct levels every other seed."""
    for seed in range(30):
        rng = np.random.default_rng(8000 + seed)
        L, n = int(rng.integers(1, 15)), int(rng.integers(1, 9))
        cf = float(rng.choice([0.4, 1.0, 2.0, 4.0]))
        w = W.random_instances(seed=8000 + seed, n_inst=5, L=L, k=min(n, L), capacity_factor=cf, quantised=seed % 2 == 1)
        if n > L:   # clusters larger than the chain: extra nodes of random capacity
            extra = n - L
            M = np.concatenate([w.M, rng.uniform(0.1, 1.0, size=(w.n_inst, extra)).astype(np.float32) * w.m.sum(axis=1, keepdims=True)], axis=1).astype(np.float32)
            B = rng.uniform(1.0, 50.0, size=(w.n_inst, n, n)).astype(np.float32)
            B = np.maximum(B, B.transpose(0, 2, 1))
            for i in range(w.n_inst):
                np.fill_diagonal(B[i], 0)
            w = Workload(w.name, L, n, w.n_inst, w.seed, w.t, w.m, M, B)
        for pmax in range(1, min(n, 8) + 1):
            print(f"few small seed={seed} L={L} n={n} pmax={pmax}", flush=True)
            got = solve_few(ppo, w, pmax)
            assert_same(got, oracle(w, pmax, CO.subset_dp), f"seed {seed} L={L} n={n} pmax={pmax}")


def test_equals_the_unused_set_form(ppo):
    """Where both formulations apply they return the same answer, element by element (n up to 16, L = 100 and 128)."""
    import torch
    for n, L, pmax in ((10, 100, 4), (12, 128, 3), (16, 100, 5), (16, 64, 2), (14, 100, 6)):
        w = W.cluster_mixed(n, L=L, n_inst=3, seed=30 + n)
        print(f"few vs unused-set form n={n} L={L} pmax={pmax}", flush=True)
        got = solve_few(ppo, w, pmax)
        ref = ppo.ppo_solve_cluster(*ppo.to_device(w), max_segments=pmax)
        torch.cuda.synchronize()
        assert_same(got, tuple(x.cpu().numpy() for x in ref), f"n={n} L={L} pmax={pmax}")
    for n, cap in ((10, 32), (15, 24), (20, 16)):
        w = W.cluster_geometric(n, cap, n_inst=4, seed=40 + n)
        for pmax in (3, 5):
            print(f"few vs unused-set form geometric n={n} pmax={pmax}", flush=True)
            got = solve_few(ppo, w, pmax)
            ref = ppo.ppo_solve_cluster(*ppo.to_device(w), max_segments=pmax)
            torch.cuda.synchronize()
            assert_same(got, tuple(x.cpu().numpy() for x in ref), f"geometric n={n} pmax={pmax}")


def test_beyond_twenty_nodes_against_the_oracle(ppo):
    """24 to 64 usable nodes, at most 2 to 4 segments: the oracle walks every node sequence."""
    for n, L, pmax, seed, cf in ((24, 40, 3, 1, 0.2), (30, 100, 2, 2, 0.3), (33, 64, 3, 3, 0.2), (40, 128, 2, 4, 0.3),
                                 (64, 30, 2, 5, 0.3), (26, 100, 4, 6, 0.15)):
        w = W.cluster_mixed(n, L=L, n_inst=2, seed=50 + seed, capacity_factor=cf)   # no node holds the whole model
        print(f"few n={n} L={L} pmax={pmax}", flush=True)
        got = solve_few(ppo, w, pmax)
        assert_same(got, oracle(w, pmax, CO.exhaustive), f"n={n} L={L} pmax={pmax}")
    # paper-shaped: 50 devices of 64 MB under the 50-layer chain (two or three partitions)
    w = W.cluster_geometric(50, 64, n_inst=3, seed=77)
    for pmax in (2, 3):
        print(f"few geometric n=50 pmax={pmax}", flush=True)
        assert_same(solve_few(ppo, w, pmax), oracle(w, pmax, CO.exhaustive), f"geometric n=50 pmax={pmax}")


def test_fifty_nodes_five_segments(ppo):
    """The paper's largest cluster with more segments than the oracle can walk sequences for: clusters of 50 and 64
    in which 8 nodes matter and the rest are too small for any layer.  The answer is the small cluster's (oracle:
    subset route), carried to the places of its nodes; every set of up to five or six of the 50 goes through the
    kernels all the same."""
    rng = np.random.default_rng(9)
    for n, L, pmax, seed in ((50, 100, 5, 0), (50, 60, 6, 1), (64, 100, 4, 2)):
        small = W.cluster_mixed(8, L=L, n_inst=2, seed=60 + seed, capacity_factor=0.3)
        big, places = with_decoys(small, n, rng)
        print(f"few decoys n={n} L={L} pmax={pmax}", flush=True)
        got = solve_few(ppo, big, pmax)
        for i in range(big.n_inst):
            beta, p, cuts, order = CO.subset_dp(small.t[i], big.m[i], small.M[i], small.B[i], pmax)
            assert bits(got[0][i]) == bits(beta) and got[1][i] == p, (n, i, got[0][i], beta, got[1][i], p)
            assert list(got[3][i][:p]) == [int(places[i][j]) for j in order[:p]] and (got[3][i][p:] == -1).all()
            assert list(got[2][i][:max(p - 1, 0)]) == list(cuts[:max(p - 1, 0)]) and (got[2][i][max(p - 1, 0):] == -1).all()
    # all 50 usable: what holds at any size
    w = W.cluster_geometric(50, 32, n_inst=2, seed=78)
    got = solve_few(ppo, w, 5)
    g3 = solve_few(ppo, w, 3)
    for i in range(w.n_inst):
        t, m, M, B = w.t[i], w.m[i], w.M[i], w.B[i]
        p = int(got[1][i])
        assert p >= 1 and bits(CO.sequence_beta(t, m, M, B, got[3][i][:p])) == bits(got[0][i])
        assert bits(got[0][i]) <= bits(g3[0][i])      # more segments allowed never hurts
        for _ in range(300):
            q = int(rng.integers(1, 6))
            seq = rng.permutation(50)[:q]
            assert bits(CO.sequence_beta(t, m, M, B, seq)) >= bits(got[0][i])


def test_workspace_size_does_not_matter_and_bad_shapes_are_refused(ppo):
    import torch
    w = W.cluster_mixed(12, L=50, n_inst=5, seed=91)
    ref = solve_few(ppo, w, 4)
    # a little less than all five need together: the rows of four fit, so the batch runs in two parts
    got = solve_few(ppo, w, 4, workspace_bytes=ppo.ppo_cluster_few_workspace_bytes(50, 12, 4, 5) - 256)
    assert_same(got, ref, "in two parts")
    assert ppo.ppo_cluster_few_workspace_bytes(100, 65, 3, 1) == 0
    assert ppo.ppo_cluster_few_workspace_bytes(100, 64, 9, 1) == 0
    assert ppo.ppo_cluster_few_workspace_bytes(100, 64, 8, 1) == 0          # more than 2^31 rows
    assert 4 * 10**8 < ppo.ppo_cluster_few_workspace_bytes(100, 50, 5, 1) < 5 * 10**8   # 982,500 rows of 400 bytes, 10.6 million words
    with pytest.raises(ppo.PpoError):
        ppo.ppo_solve_cluster_few(*ppo.to_device(w), max_segments=13)
    with pytest.raises(ppo.PpoError):
        ppo.ppo_solve_cluster_few(*ppo.to_device(w), max_segments=4, workspace=torch.empty(1024, dtype=torch.uint8, device="cuda:0"))
