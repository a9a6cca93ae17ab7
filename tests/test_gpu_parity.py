"""Parity of the HIP path (through the C ABI) with the CPU oracle, bit for bit: beta, cuts, ordering."""
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


def gpu_solve(ppo, w, **kw):
    import torch
    dev = ppo.to_device(w)
    beta, cuts, order = ppo.ppo_solve(*dev, **kw)
    torch.cuda.synchronize()
    return beta.cpu().numpy(), cuts.cpu().numpy(), order.cpu().numpy()


def assert_same(got, ref, what=""):
    bad = np.nonzero(bits(got[0]) != bits(ref[0]))[0]
    assert bad.size == 0, f"{what}: beta differs at instances {bad[:8]}: {got[0][bad[:4]]} vs {ref[0][bad[:4]]}"
    assert np.array_equal(got[2], ref[2]), f"{what}: ordering differs"
    assert np.array_equal(got[1], ref[1]), f"{what}: cuts differ"


def test_worked_example(ppo):
    """Sec. I: 10.2 Mbit over 6 Mbps, about 1.7 s; binary32 quotient 0x3FD99999."""
    w = W.Workload("ex", 2, 2, 1, 0, np.array([[10.2, 3.0]], np.float32), np.ones((1, 2), np.float32),
                   np.full((1, 2), 5.0, np.float32), np.array([[[0, 6], [6, 0]]], np.float32))
    beta, cuts, order = gpu_solve(ppo, w)
    assert int(bits(beta)[0]) == 0x3FD99999 and cuts.tolist() == [[1]] and order.tolist() == [[0, 1]]


def test_tiny_workload_against_brute_force_and_exhaustive(ppo):
    w = W.tiny()
    got = gpu_solve(ppo, w)
    assert_same(got, O.bruteforce(w.t, w.m, w.M, w.B), "tiny vs brute force")
    assert_same(got, O.exhaustive(w.t, w.m, w.M, w.B)[:3], "tiny vs exhaustive")
    assert np.isinf(got[0]).sum() > 10          # the workload does contain infeasible instances


def test_per_ordering_beta_tiny_and_resnet(ppo):
    import torch
    for w, n in ((W.tiny(), 24), (W.resnet50_shaped(), 6)):
        dev = ppo.to_device(w.take(n))
        kf = math.factorial(w.k)
        for j in range(n):
            got = ppo.ppo_eval_orderings(dev[0][j], dev[1][j], dev[2][j], dev[3][j], 0, kf)
            torch.cuda.synchronize()
            ref, _ = O.eval_orderings(w.t[j], w.m[j], w.M[j], w.B[j], 0, kf)
            assert np.array_equal(bits(got.cpu().numpy()), bits(ref)), (w.name, j)


def test_resnet_workload_full(ppo):
    w = W.resnet50_shaped()
    assert_same(gpu_solve(ppo, w), O.exhaustive(w.t, w.m, w.M, w.B)[:3], "resnet50_shaped")


def test_transformer_workload_full(ppo):
    """Almost every ordering ties on beta here: this is the test of the lowest-rank rule."""
    w = W.transformer_encoder()
    got = gpu_solve(ppo, w)
    assert_same(got, O.subset_dp(w.t, w.m, w.M, w.B), "transformer vs subset DP")
    head = w.take(8)
    assert_same(tuple(x[:8] for x in got), O.exhaustive(head.t, head.m, head.M, head.B)[:3],
                "transformer vs exhaustive")


def sampled_orderings_match(ppo, w, inst, n_ranges, width, seed):
    import torch
    rng = np.random.default_rng(seed)
    kf = math.factorial(w.k)
    dev = ppo.to_device(w)
    for j in inst:
        for _ in range(n_ranges):
            r0 = int(rng.integers(0, kf - width))
            got = ppo.ppo_eval_orderings(dev[0][j], dev[1][j], dev[2][j], dev[3][j], r0, r0 + width)
            torch.cuda.synchronize()
            ref, _ = O.eval_orderings(w.t[j], w.m[j], w.M[j], w.B[j], r0, r0 + width)
            assert np.array_equal(bits(got.cpu().numpy()), bits(ref)), (w.name, j, r0)


def test_headline_workload_full(ppo):
    """Full size, in the launch configuration the benchmark times: the optimum against the independent
    subset DP, plus beta of sampled orderings one by one against the per-ordering oracle."""
    w = W.headline()
    got = gpu_solve(ppo, w)
    assert_same(got, O.subset_dp(w.t, w.m, w.M, w.B), "headline vs subset DP")
    sampled_orderings_match(ppo, w, [0, 17, 63], 3, 3000, seed=1)


def test_headline_in_two_ragged_pieces(ppo):
    """The headline search cut at a rank inside a group of orderings: the large piece starts ragged and is
    long enough for the launch shape with more groups per workgroup; the pieces' common key is the whole
    search's, checked against the independent subset DP."""
    import torch
    w = W.headline()
    dev = ppo.to_device(w)
    ws = ppo.alloc_workspace(w.L, w.k, w.n_inst)
    keys = torch.empty(w.n_inst, dtype=torch.int64, device="cuda:0")
    ppo.ppo_prepare(*dev, ws)
    ppo.ppo_init_keys(keys)
    cut = 16 * 720 + 257
    for a, b in ((cut, math.factorial(w.k)), (0, cut)):
        ppo.ppo_solve_range(w.L, w.k, w.n_inst, ws, a, b, keys)
    out = ppo.ppo_finalize(w.L, w.k, w.n_inst, ws, keys)
    torch.cuda.synchronize()
    assert_same(tuple(x.cpu().numpy() for x in out), O.subset_dp(w.t, w.m, w.M, w.B), "headline in two pieces")


def test_headline_in_both_launch_shapes(ppo):
    """The enumeration launch gives a workgroup 16 groups of orderings where the grid stays large (all 64
    headline instances at once: 5040 / 16 * 2 * 64 = 40,320 workgroups) and 8 otherwise (16 instances at a
    time: 10,080 workgroups of 16 groups would be fewer than 16,384).  Both shapes over the whole rank range
    must leave the same keys, and they are the subset DP's."""
    import torch
    w = W.headline()
    kf = math.factorial(w.k)
    assert (kf // 720) % 16 == 0 and (kf // 720 // 16) * 2 * 64 >= 16384 > (kf // 720 // 16) * 2 * 16
    dev = ppo.to_device(w)
    ws = ppo.alloc_workspace(w.L, w.k, w.n_inst)
    ppo.ppo_prepare(*dev, ws)
    keys16 = torch.empty(w.n_inst, dtype=torch.int64, device="cuda:0")
    ppo.ppo_init_keys(keys16)
    ppo.ppo_solve_range(w.L, w.k, w.n_inst, ws, 0, kf, keys16)
    keys8 = torch.empty(w.n_inst, dtype=torch.int64, device="cuda:0")
    ppo.ppo_init_keys(keys8)
    for first in range(0, w.n_inst, 16):
        part = tuple(x[first:first + 16].contiguous() for x in dev)
        ws_part = ppo.alloc_workspace(w.L, w.k, 16)
        ppo.ppo_prepare(*part, ws_part)
        ppo.ppo_solve_range(w.L, w.k, 16, ws_part, 0, kf, keys8[first:first + 16])
    torch.cuda.synchronize()
    assert np.array_equal(keys16.cpu().numpy(), keys8.cpu().numpy())
    ref = O.subset_dp(w.t, w.m, w.M, w.B)
    k16 = keys16.cpu().numpy().view(np.uint64)
    assert np.array_equal((k16 >> np.uint64(32)).astype(np.uint32), bits(ref[0]))
    want_rank = np.array([O.rank(ref[2][i]) for i in range(w.n_inst)], np.uint64)
    assert np.array_equal(k16 & np.uint64(0xFFFFFFFF), want_rank)


def test_paired_and_grouped_kernels_at_twelve_nodes(ppo):
    """k = 12 with rows short enough for the paired and the grouped kernel (L - k + 2 <= 96): six prefix digits,
    five links inside the prefix, four kept prefix rows in the bounded mode.  Ragged rank ranges at both ends of
    [0, 12!) through every route that takes a range, against the oracle on the same ranges, with each kernel."""
    import torch
    kf = math.factorial(12)
    for seed, L in ((1, 30), (2, 47), (3, 60)):
        w = W.random_instances(1200 + seed, 2, L, 12, capacity_factor=1.3 + 0.1 * seed)
        dev = ppo.to_device(w)
        ws = ppo.alloc_workspace(L, 12, 2)
        ppo.ppo_prepare(*dev, ws)
        for r0, r1 in ((0, 30011), (kf - 25013, kf), (kf // 2 - 977, kf // 2 + 20000)):
            ref = O.exhaustive(w.t, w.m, w.M, w.B, rank_range=(r0, r1))[:3]
            per = [O.eval_orderings(w.t[j], w.m[j], w.M[j], w.B[j], r0, min(r1, r0 + 6000))[0] for j in range(2)]
            for variant in (ppo.PPO_ENUM_AUTO, ppo.PPO_ENUM_GROUPED):
                print(f"k=12 L={L} ranks [{r0}, {r1}) kernel {variant}", flush=True)
                try:
                    ppo.ppo_set_enumeration(variant)
                    for bounded in (False, True):
                        keys = torch.empty(2, dtype=torch.int64, device="cuda:0")
                        ppo.ppo_init_keys(keys)
                        if bounded:
                            ppo.ppo_solve_range_bounded(L, 12, 2, ws, r0, r1, keys, None)
                        else:
                            ppo.ppo_solve_range(L, 12, 2, ws, r0, r1, keys)
                        out = tuple(x.cpu().numpy() for x in ppo.ppo_finalize(L, 12, 2, ws, keys))
                        torch.cuda.synchronize()
                        assert_same(out, ref, f"k=12 L={L} [{r0},{r1}) bounded={bounded} kernel {variant}")
                    for j in range(2):
                        a, b = r0, min(r1, r0 + 6000)
                        got = ppo.ppo_eval_orderings(dev[0][j], dev[1][j], dev[2][j], dev[3][j], a, b)
                        torch.cuda.synchronize()
                        assert np.array_equal(bits(got.cpu().numpy()), bits(per[j])), (L, j, a, variant)
                finally:
                    ppo.ppo_set_enumeration(ppo.PPO_ENUM_AUTO)


def test_large_workload_full(ppo):
    w = W.large()
    got = gpu_solve(ppo, w)
    assert np.isfinite(got[0][0])
    assert_same(got, O.subset_dp(w.t, w.m, w.M, w.B), "large vs subset DP")
    sampled_orderings_match(ppo, w, [0], 4, 5000, seed=2)


def test_small_instances_with_ties_and_exact_capacity_hits(ppo):
    for seed in range(24):
        rng = np.random.default_rng(5000 + seed)
        L = int(rng.integers(1, 11))
        k = int(rng.integers(1, min(L, 5) + 1))
        w = W.random_instances(seed, 50, L, k, capacity_factor=float(rng.uniform(1.0, 1.8)), quantised=bool(seed % 2))
        ref = O.exhaustive(w.t, w.m, w.M, w.B)[:3] if k == 5 else O.bruteforce(w.t, w.m, w.M, w.B)
        assert_same(gpu_solve(ppo, w), ref, f"random L={L} k={k} seed={seed}")


def test_degenerate_shapes(ppo):
    # k = 1
    w = W.random_instances(1, 9, 7, 1, capacity_factor=1.2)
    w.M[::2] *= np.float32(0.5)                     # every other instance cannot hold the model
    got = gpu_solve(ppo, w)
    assert_same(got, O.bruteforce(w.t, w.m, w.M, w.B), "k=1")
    assert np.isinf(got[0][::2]).all() and (got[0][1::2] == 0).all()
    # L = k: every segment is a single layer
    w = W.random_instances(2, 40, 5, 5, capacity_factor=3.0)
    assert_same(gpu_solve(ppo, w), O.bruteforce(w.t, w.m, w.M, w.B), "L=k")
    # L = k = 1
    w = W.random_instances(3, 4, 1, 1, capacity_factor=1.5)
    assert_same(gpu_solve(ppo, w), O.bruteforce(w.t, w.m, w.M, w.B), "L=k=1")
    # nothing fits anywhere
    w = W.random_instances(4, 5, 9, 3, capacity_factor=0.5)
    got = gpu_solve(ppo, w)
    assert np.isinf(got[0]).all() and (got[1] == -1).all() and (got[2] == -1).all()
    # zero transfer sizes are legal and give beta = +0
    w = W.random_instances(5, 3, 6, 3, capacity_factor=3.0)
    w.t[:] = 0
    got = gpu_solve(ppo, w)
    assert (bits(got[0]) == 0).all()
    assert_same(got, O.bruteforce(w.t, w.m, w.M, w.B), "t=0")
    # a zero with the sign bit set is a size of zero too: gamma = +0, never the bit pattern of -0
    w = W.random_instances(6, 30, 7, 3, capacity_factor=2.0)
    w.t[:, ::2] = np.float32(-0.0)
    assert np.signbit(w.t).any()
    got = gpu_solve(ppo, w)
    ref = O.bruteforce(w.t, w.m, w.M, w.B)
    assert not (bits(ref[0]) == 0x80000000).any() and (bits(ref[0]) == 0).any()
    assert_same(got, ref, "t=-0")
    plus = W.Workload(w.name, w.L, w.k, w.n_inst, w.seed, np.abs(w.t), w.m, w.M, w.B)
    assert_same(got, O.bruteforce(plus.t, plus.m, plus.M, plus.B), "t=-0 against t=+0")


def test_memory_rule_in_binary64(ppo):
    """Sums of weights near 2^24, where binary32 sums or a binary32 comparison would let a segment of
    2^24 + 1 into a node of 2^24: every stage-2 route against the oracle's definition route."""
    import torch
    big = np.float32(2.0 ** 24)
    rng = np.random.default_rng(77)
    L, k, n = 6, 3, 64
    t = rng.integers(1, 9, (n, L)).astype(np.float32)
    m = rng.choice(np.array([1, 2, 3, big, big + np.float32(2)], np.float32), (n, L), p=[0.3, 0.2, 0.2, 0.2, 0.1])
    M = rng.choice(np.array([big, big + np.float32(2), big + np.float32(4), 4], np.float32), (n, k))
    B = np.ones((n, k, k), np.float32)
    w = W.Workload("near 2^24", L, k, n, 77, t, m, M, B)
    ref = O.bruteforce(w.t, w.m, w.M, w.B)
    assert np.isfinite(ref[0]).sum() >= 8 and np.isinf(ref[0]).sum() >= 8
    assert_same(gpu_solve(ppo, w), ref, "near 2^24")
    dev = ppo.to_device(w)
    ws = ppo.alloc_workspace(L, k, n)
    for route in ("bounded", "subsets"):
        keys = torch.empty(n, dtype=torch.int64, device="cuda:0")
        ppo.ppo_prepare(*dev, ws)
        ppo.ppo_init_keys(keys)
        if route == "bounded":
            ppo.ppo_solve_range_bounded(L, k, n, ws, 0, math.factorial(k), keys, None)
        else:
            ppo.ppo_solve_subsets(L, k, n, ws, keys)
        out = tuple(x.cpu().numpy() for x in ppo.ppo_finalize(L, k, n, ws, keys))
        torch.cuda.synchronize()
        assert_same(out, ref, f"near 2^24, {route}")


def test_empty_batch(ppo):
    import torch
    z = lambda *s: torch.zeros(s, dtype=torch.float32, device="cuda:0")
    beta, cuts, order = ppo.ppo_solve(z(0, 5), z(0, 5), z(0, 3), z(0, 3, 3))
    torch.cuda.synchronize()
    assert beta.numel() == 0 and cuts.shape == (0, 2) and order.shape == (0, 3)


def test_maximum_sizes_on_a_rank_range(ppo):
    """L = 128, k = 12 (the compiled limits): 12! orderings is too many to enumerate in a test, so a rank
    range goes through solve_range + finalize and is compared with the oracle on the same range."""
    import torch
    w = W.random_instances(77, 2, 128, 12, capacity_factor=1.3)
    dev = ppo.to_device(w)
    kf = math.factorial(12)
    r0, r1 = kf - 70001, kf
    ws = ppo.alloc_workspace(128, 12, 2)
    keys = torch.empty(2, dtype=torch.int64, device="cuda:0")
    ppo.ppo_prepare(*dev, ws)
    ppo.ppo_init_keys(keys)
    ppo.ppo_solve_range(128, 12, 2, ws, r0, r1, keys)
    beta, cuts, order = ppo.ppo_finalize(128, 12, 2, ws, keys)
    torch.cuda.synchronize()
    ref = O.exhaustive(w.t, w.m, w.M, w.B, rank_range=(r0, r1))[:3]
    assert_same((beta.cpu().numpy(), cuts.cpu().numpy(), order.cpu().numpy()), ref, "L=128 k=12 range")
    j = 1
    got = ppo.ppo_eval_orderings(dev[0][j], dev[1][j], dev[2][j], dev[3][j], r1 - 3000, r1)
    torch.cuda.synchronize()
    per, _ = O.eval_orderings(w.t[j], w.m[j], w.M[j], w.B[j], r1 - 3000, r1)
    assert np.array_equal(bits(got.cpu().numpy()), bits(per))


def test_rank_ranges_compose_and_workspace_variant(ppo):
    """Ragged pieces of the rank range, issued out of order, give the key of the whole search; and the
    caller-workspace entry point equals the allocating one."""
    import torch
    w = W.resnet50_shaped().take(37)
    dev = ppo.to_device(w)
    whole = gpu_solve(ppo, w)
    ws = ppo.alloc_workspace(w.L, w.k, w.n_inst)
    assert_same(gpu_solve(ppo, w, workspace=ws), whole, "workspace variant")
    keys = torch.empty(w.n_inst, dtype=torch.int64, device="cuda:0")
    ppo.ppo_prepare(*dev, ws)
    ppo.ppo_init_keys(keys)
    for a, b in ((301, 720), (0, 1), (64, 301), (1, 64), (5, 5)):
        ppo.ppo_solve_range(w.L, w.k, w.n_inst, ws, a, b, keys)
    out = ppo.ppo_finalize(w.L, w.k, w.n_inst, ws, keys)
    torch.cuda.synchronize()
    assert_same(tuple(x.cpu().numpy() for x in out), whole, "composed ranges")


def test_division_is_correctly_rounded_on_a_million_pairs(ppo):
    """k = 2, L = 2 with ample memory reduces the search to one quotient t[0]/B[0][1] (Eq. 3)."""
    n = 1_000_000
    rng = np.random.default_rng(123)
    t0 = np.exp(rng.uniform(np.log(1e-6), np.log(1e6), n)).astype(np.float32)
    b = np.exp(rng.uniform(np.log(1e-3), np.log(1e5), n)).astype(np.float32)
    t = np.stack([t0, np.ones(n, np.float32)], 1)
    B = np.zeros((n, 2, 2), np.float32)
    B[:, 0, 1] = B[:, 1, 0] = b
    w = W.Workload("div", 2, 2, n, 0, np.ascontiguousarray(t), np.ones((n, 2), np.float32),
                   np.full((n, 2), 8.0, np.float32), B)
    beta, cuts, order = gpu_solve(ppo, w)
    assert np.array_equal(bits(beta), bits(t0 / b))
    assert (cuts == 1).all() and (order == np.array([0, 1])).all()


def test_grouped_kernel_row_lengths(ppo):
    """The grouped kernel cuts a row of NP = ceil((L-k+2)/2) output dwords into one to four parts of three
    chunks: sweep NP from 1 to its maximum of 48 (and one past it, which goes to the generic kernel), with
    k = 6, 7 and 9, against the subset DP."""
    cases = [(6, 6), (6, 7), (6, 9), (6, 13), (6, 27), (6, 28), (6, 29), (6, 51), (6, 52), (6, 53), (6, 75),
             (6, 76), (6, 77), (6, 99), (6, 100), (6, 101), (7, 7), (7, 30), (7, 54), (7, 78), (7, 101), (7, 102),
             (9, 9), (9, 20), (9, 57), (9, 103)]
    for n, (k, L) in enumerate(cases):
        w = W.random_instances(7000 + n, 3 if k == 9 else 10, L, k, capacity_factor=1.15 + 0.1 * (n % 4),
                               quantised=bool(n % 3 == 0))
        assert_same(gpu_solve(ppo, w), O.subset_dp(w.t, w.m, w.M, w.B), f"grouped row lengths k={k} L={L}")


def test_grouped_kernel_behind_the_switch(ppo):
    """The grouped kernel (one ordering per lane, rows in LDS) is what the bounded search runs and what
    PPO_ENUM_GROUPED selects: with the switch set, the headline keys, row lengths at its part boundaries, k = 12 and
    per-ordering values, against the oracle."""
    import torch
    ppo.ppo_set_enumeration(ppo.PPO_ENUM_GROUPED)
    try:
        w = W.headline()
        assert_same(gpu_solve(ppo, w), O.subset_dp(w.t, w.m, w.M, w.B), "headline, grouped kernel")
        sampled_orderings_match(ppo, w, [5], 2, 3000, seed=7)
        for n, (k, L) in enumerate([(6, 6), (6, 28), (6, 29), (6, 53), (6, 77), (6, 100), (7, 54), (9, 57), (9, 103)]):
            w = W.random_instances(7100 + n, 4, L, k, capacity_factor=1.15 + 0.1 * (n % 4), quantised=bool(n % 3 == 0))
            assert_same(gpu_solve(ppo, w), O.subset_dp(w.t, w.m, w.M, w.B), f"grouped kernel k={k} L={L}")
        kf = math.factorial(12)
        w = W.random_instances(1299, 1, 40, 12, capacity_factor=1.4)
        dev = ppo.to_device(w)
        r0, r1 = kf - 9000, kf
        got = ppo.ppo_eval_orderings(dev[0][0], dev[1][0], dev[2][0], dev[3][0], r0, r1)
        torch.cuda.synchronize()
        per, _ = O.eval_orderings(w.t[0], w.m[0], w.M[0], w.B[0], r0, r1)
        assert np.array_equal(bits(got.cpu().numpy()), bits(per))
    finally:
        ppo.ppo_set_enumeration(ppo.PPO_ENUM_AUTO)


def test_issue_probe_runs(ppo):
    """The measurement aid launches and keeps its work: every lane writes the sum of its eight accumulators."""
    import torch
    for wps in (1, 4):
        sink = torch.full((256 * 256 * wps,), -1, dtype=torch.int32, device="cuda:0")
        ppo.ppo_probe_valu(wps, 10, sink)
        torch.cuda.synchronize()
        got = sink.cpu().numpy().view(np.uint32).reshape(256, 256 * wps)
        # by hand: a = min(max(a, x), y) halfword by halfword settles after one round
        tid = np.arange(256 * wps, dtype=np.uint32)[None, :]
        blk = np.arange(256, dtype=np.uint32)[:, None]
        x = (blk * np.uint32(0x00010001) + np.uint32(0x00030005)).astype(np.uint32)
        yv = (np.uint32(0x7F007F00) ^ tid).astype(np.uint32)

        def halves(v):
            return (v & np.uint32(0xFFFF)).astype(np.uint32), (v >> np.uint32(16)).astype(np.uint32)

        def clamp(a):
            out = np.zeros(np.broadcast(a, x, yv).shape, np.uint32)
            for h, (ah, xh, yh) in enumerate(zip(halves(a), halves(x), halves(yv))):
                out |= (np.minimum(np.maximum(ah, xh), yh).astype(np.uint32) << np.uint32(16 * h))
            return out

        want = np.zeros((256, 256 * wps), np.uint32)
        for mul in (1, 3, 5, 7, 11, 13, 17, 19):
            want = (want + clamp((tid * np.uint32(mul)).astype(np.uint32))).astype(np.uint32)
        assert np.array_equal(got, want)

