"""The shared-prefix, bounded enumeration (ppo_solve_range_bounded) against the CPU oracle and against the
full enumeration: same beta, cuts and ordering bit for bit, same keys; it only does less work."""
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


def solve_bounded(ppo, w, ranges=None):
    """(beta, cuts, order), keys, skipped groups per instance"""
    import torch
    dev = ppo.to_device(w)
    ws = ppo.alloc_workspace(w.L, w.k, w.n_inst)
    keys = torch.empty(w.n_inst, dtype=torch.int64, device="cuda:0")
    skipped = torch.zeros(w.n_inst, dtype=torch.int64, device="cuda:0")
    ppo.ppo_prepare(*dev, ws)
    ppo.ppo_init_keys(keys)
    for a, b in (ranges or [(0, math.factorial(w.k))]):
        ppo.ppo_solve_range_bounded(w.L, w.k, w.n_inst, ws, a, b, keys, skipped)
    out = ppo.ppo_finalize(w.L, w.k, w.n_inst, ws, keys)
    torch.cuda.synchronize()
    return tuple(x.cpu().numpy() for x in out), keys.cpu().numpy(), skipped.cpu().numpy()


def solve_full_keys(ppo, w):
    import torch
    dev = ppo.to_device(w)
    ws = ppo.alloc_workspace(w.L, w.k, w.n_inst)
    keys = torch.empty(w.n_inst, dtype=torch.int64, device="cuda:0")
    ppo.ppo_prepare(*dev, ws)
    ppo.ppo_init_keys(keys)
    ppo.ppo_solve_range(w.L, w.k, w.n_inst, ws, 0, math.factorial(w.k), keys)
    torch.cuda.synchronize()
    return keys.cpu().numpy()


def assert_same(got, ref, what=""):
    bad = np.nonzero(bits(got[0]) != bits(ref[0]))[0]
    assert bad.size == 0, f"{what}: beta differs at instances {bad[:8]}: {got[0][bad[:4]]} vs {ref[0][bad[:4]]}"
    assert np.array_equal(got[2], ref[2]), f"{what}: ordering differs"
    assert np.array_equal(got[1], ref[1]), f"{what}: cuts differ"


def test_headline_bounded(ppo):
    w = W.headline()
    got, keys, skipped = solve_bounded(ppo, w)
    assert_same(got, O.subset_dp(w.t, w.m, w.M, w.B), "headline, bounded vs subset DP")
    assert np.array_equal(keys, solve_full_keys(ppo, w)), "keys differ from the full enumeration"
    groups = math.factorial(w.k) // 360
    assert (skipped >= 0).all() and (skipped <= groups).all()
    assert skipped.sum() > 0          # the bound does bite on this workload


def test_transformer_bounded_ties(ppo):
    """Nearly every ordering ties here: a group may only be skipped when it cannot even tie."""
    w = W.transformer_encoder()
    got, keys, _ = solve_bounded(ppo, w)
    assert_same(got, O.subset_dp(w.t, w.m, w.M, w.B), "transformer, bounded vs subset DP")
    assert np.array_equal(keys, solve_full_keys(ppo, w))


def test_large_bounded(ppo):
    w = W.large()
    got, keys, _ = solve_bounded(ppo, w)
    assert_same(got, O.subset_dp(w.t, w.m, w.M, w.B), "large, bounded vs subset DP")
    assert np.array_equal(keys, solve_full_keys(ppo, w))


def test_bounded_small_and_ragged(ppo):
    """k = 7 (a prefix of one node), k = 6 and k < 6 (no prefix: evaluated in full), infeasible-heavy and
    quantised instances, and ragged rank ranges out of order."""
    for seed, (L, k, cap, q) in enumerate([(12, 7, 1.3, True), (20, 7, 1.1, False), (16, 8, 1.2, True),
                                           (14, 6, 1.3, True), (9, 4, 1.4, False), (30, 9, 1.05, True)]):
        w = W.random_instances(900 + seed, 12 if k >= 8 else 40, L, k, capacity_factor=cap, quantised=q)
        ref = O.subset_dp(w.t, w.m, w.M, w.B)
        got, keys, _ = solve_bounded(ppo, w)
        assert_same(got, ref, f"bounded L={L} k={k}")
        assert np.array_equal(keys, solve_full_keys(ppo, w)), (L, k)
        kf = math.factorial(k)
        cuts = sorted({0, kf, kf // 3 + 1, kf // 2 + 7, min(kf, 361), min(kf, 1000)})
        pieces = list(zip(cuts[:-1], cuts[1:]))[::-1]
        got2, keys2, _ = solve_bounded(ppo, w, ranges=pieces)
        assert_same(got2, ref, f"bounded, ragged ranges L={L} k={k}")
        assert np.array_equal(keys2, keys)


def test_bounded_row_lengths(ppo):
    """Row lengths from one dword to the maximum, prefixes of one to three nodes."""
    cases = [(7, 7), (7, 8), (7, 31), (7, 55), (7, 79), (7, 101), (7, 102), (8, 8), (8, 33), (8, 80), (8, 102),
             (9, 9), (9, 58), (9, 103)]
    for n, (k, L) in enumerate(cases):
        w = W.random_instances(8000 + n, 3 if k == 9 else 8, L, k, capacity_factor=1.1 + 0.1 * (n % 4),
                               quantised=bool(n % 2))
        # The kernel must not depend on what an earlier kernel left in LDS (it once read a row buffer it had
        # not written yet).  Best effort: sorting and scanning all-ones words leaves 0xFFFF patterns, which no
        # order code ever is, in the LDS of many compute units.
        import torch
        junk = torch.full((1 << 22,), -1, dtype=torch.int32, device="cuda:0")
        junk.sort()
        torch.cumsum(junk.view(1 << 11, 1 << 11), dim=1)
        got, keys, _ = solve_bounded(ppo, w)
        assert_same(got, O.subset_dp(w.t, w.m, w.M, w.B), f"bounded row lengths k={k} L={L}")
        assert np.array_equal(keys, solve_full_keys(ppo, w)), (k, L)


def test_bounded_mode_of_the_grouped_kernel_behind_the_switch(ppo):
    """ppo_solve_range_bounded runs the paired kernel where it applies; the grouped kernel's bounded mode stays
    reachable through ppo_set_enumeration and must leave the same keys."""
    w = W.random_instances(950, 16, 40, 8, capacity_factor=1.2, quantised=True)
    ref_keys = solve_full_keys(ppo, w)
    try:
        ppo.ppo_set_enumeration(ppo.PPO_ENUM_GROUPED)
        got, keys, skipped = solve_bounded(ppo, w)
    finally:
        ppo.ppo_set_enumeration(ppo.PPO_ENUM_AUTO)
    assert np.array_equal(keys, ref_keys)
    assert_same(got, O.subset_dp(w.t, w.m, w.M, w.B), "grouped kernel, bounded")
    got2, keys2, skipped2 = solve_bounded(ppo, w)
    assert np.array_equal(keys2, ref_keys)
