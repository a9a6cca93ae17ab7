"""The search with the compute-time term (ppo_solve_ct; Sec. I, Eq. 1) through the C ABI against its CPU oracle,
bit for bit: beta, cuts, ordering."""
import math

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import ppo_ct_oracle as CT
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


def gpu_solve(ppo, w, work, speed):
    import torch
    t, m, M, B = ppo.to_device(w)
    out = ppo.ppo_solve_ct(t, m, torch.from_numpy(work).cuda(), M, torch.from_numpy(speed).cuda(), B)
    torch.cuda.synchronize()
    return tuple(x.cpu().numpy() for x in out)


def oracle(w, work, speed, route, idx=None):
    idx = range(w.n_inst) if idx is None else idx
    res = [route(w.t[i], w.m[i], work[i], w.M[i], speed[i], w.B[i]) for i in idx]
    return (np.array([r[0] for r in res], np.float32), np.array([r[1] for r in res], np.int32).reshape(len(res), -1),
            np.array([r[2] for r in res], np.int32))


def assert_same(got, ref, what, idx=None):
    g = got if idx is None else tuple(x[list(idx)] for x in got)
    bad = np.nonzero(bits(g[0]) != bits(ref[0]))[0]
    assert bad.size == 0, f"{what}: beta differs at {bad[:8]}: {g[0][bad[:4]]} vs {ref[0][bad[:4]]}"
    assert np.array_equal(g[2], ref[2]), f"{what}: ordering differs"
    assert np.array_equal(g[1].reshape(ref[1].shape), ref[1]), f"{what}: cuts differ"


def test_small_shapes_ties_and_infeasible(ppo):
    for seed in range(30):
        rng = np.random.default_rng(4000 + seed)
        L = int(rng.integers(1, 11))
        k = int(rng.integers(1, min(L, 5) + 1))
        w = W.random_instances(seed, 40, L, k, capacity_factor=float(rng.uniform(1.0, 1.8)), quantised=bool(seed % 2))
        work, speed = W.compute_terms(w, seed=seed, seconds=float(rng.uniform(0.1, 8.0)), quantised=bool(seed % 3 == 0))
        print(f"ct small seed={seed} L={L} k={k}", flush=True)
        ref = oracle(w, work, speed, CT.bruteforce if k < 5 else CT.exhaustive)
        assert_same(gpu_solve(ppo, w, work, speed), ref, f"ct L={L} k={k} seed={seed}")


def test_without_work_it_is_ppo_solve(ppo):
    import torch
    for w in (W.tiny(), W.resnet50_shaped(n_inst=64), W.random_instances(5, 20, 9, 4, quantised=True)):
        work = np.zeros((w.n_inst, w.L), np.float32)
        _, speed = W.compute_terms(w)
        got = gpu_solve(ppo, w, work, speed)
        ref = tuple(x.cpu().numpy() for x in ppo.ppo_solve(*ppo.to_device(w)))
        torch.cuda.synchronize()
        assert_same(got, ref, f"zero work on {w.name}")


def test_named_workloads(ppo):
    """The five workloads with compute stages of the same magnitude as their transfers: the small ones whole,
    the large ones on a few instances (the per-ordering path is a plain one) against the subset DP."""
    import torch
    for w, seconds, n in ((W.tiny(), 1.0, None), (W.resnet50_shaped(), 2.0, 128), (W.transformer_encoder(), 10.0, 6),
                          (W.headline(), 0.5, 2), (W.large(), 2.0, 1)):
        w = w if n is None else w.take(n)
        work, speed = W.compute_terms(w, seed=11, seconds=seconds)
        print(f"ct workload {w.name} x {w.n_inst}", flush=True)
        got = gpu_solve(ppo, w, work, speed)
        ref = oracle(w, work, speed, CT.subset_dp)
        assert_same(got, ref, w.name)
        assert np.isfinite(ref[0]).any()
        base = O.subset_dp(w.t, w.m, w.M, w.B)[0]
        assert (bits(ref[0]) >= bits(base)).all() and (bits(ref[0]) > bits(base)).any()   # the stages do bind


def test_sampled_orderings_at_full_size(ppo):
    import torch
    rng = np.random.default_rng(3)
    for w, seconds in ((W.headline(), 4.0), (W.large(), 2.0), (W.random_instances(9, 2, 128, 12, capacity_factor=1.3), 3.0)):
        work, speed = W.compute_terms(w, seed=12, seconds=seconds)
        kf = math.factorial(w.k)
        dev = ppo.to_device(w)
        wd, vd = torch.from_numpy(work).cuda(), torch.from_numpy(speed).cuda()
        for j in (0, w.n_inst - 1):
            for _ in range(2):
                r0 = int(rng.integers(0, kf - 4000))
                print(f"ct per ordering {w.name} L={w.L} k={w.k} inst={j} ranks [{r0}, {r0 + 4000})", flush=True)
                got = ppo.ppo_eval_orderings_ct(dev[0][j], dev[1][j], wd[j], dev[2][j], vd[j], dev[3][j], r0, r0 + 4000)
                torch.cuda.synchronize()
                ref = CT.eval_orderings(w.t[j], w.m[j], work[j], w.M[j], speed[j], w.B[j], r0, r0 + 4000)
                assert np.array_equal(bits(got.cpu().numpy()), bits(ref)), (w.name, j, r0)


def test_degenerate_and_bad_arguments(ppo):
    import ctypes as C
    import torch
    # k = 1, L = 1, empty batch
    for L, k in ((1, 1), (5, 1), (4, 4)):
        w = W.random_instances(70 + L, 6, L, k, capacity_factor=2.0)
        work, speed = W.compute_terms(w, seed=L)
        assert_same(gpu_solve(ppo, w, work, speed), oracle(w, work, speed, CT.bruteforce), f"L={L} k={k}")
    z = lambda *s: torch.zeros(s, dtype=torch.float32, device="cuda:0")
    beta, cuts, order = ppo.ppo_solve_ct(z(0, 5), z(0, 5), z(0, 5), z(0, 3), z(0, 3), z(0, 3, 3))
    assert beta.numel() == 0
    lib, p, s = ppo.load(), C.c_void_p(0x1000), C.c_void_p(0)
    assert lib.ppo_solve_ct(p, p, None, 4, p, p, p, 2, 1, p, p, p, s) == ppo.PPO_EINVAL
    assert lib.ppo_solve_ct(p, p, p, 4, p, p, p, 5, 1, p, p, p, s) == ppo.PPO_EINVAL
    assert lib.ppo_solve_ct(p, p, p, 129, p, p, p, 5, 1, p, p, p, s) == ppo.PPO_ETOOBIG
