"""The C-ABI library: it loads, exports every entry point the header declares, and rejects bad
arguments before touching the GPU (so these run without one)."""
import ctypes as C
import os
import re

import pytest

from paper_2210_12219_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2210_12219_amd import build
        build.build()
    return binding.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ppo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ppo_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"ppo_solve", "ppo_solve_ws", "ppo_prepare", "ppo_solve_range", "ppo_solve_range_bounded", "ppo_solve_subsets", "ppo_finalize", "ppo_eval_orderings", "ppo_init_keys",
            "ppo_workspace_bytes", "ppo_strerror", "ppo_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_messages(lib):
    assert lib.ppo_version() >= 100
    assert binding.ppo_strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert binding.ppo_strerror(code)


def test_workspace_bytes(lib):
    assert binding.ppo_workspace_bytes(0, 1, 1) == 0
    assert binding.ppo_workspace_bytes(4, 5, 1) == 0          # k > L
    assert binding.ppo_workspace_bytes(129, 4, 1) == 0        # L too large
    assert binding.ppo_workspace_bytes(100, 13, 1) == 0       # k too large
    one = binding.ppo_workspace_bytes(100, 10, 1)
    many = binding.ppo_workspace_bytes(100, 10, 64)
    assert one >= 10 * 101 + 45 * 100 * 2 + (45 * 99 + 2) * 4
    assert many >= 64 * (one - 256) and many % 256 == 0


def test_bad_arguments_are_refused_without_a_gpu(lib):
    p = C.c_void_p(0x1000)     # never dereferenced: every call below must fail on its scalars first
    null = C.c_void_p(0)
    s = C.c_void_p(0)
    # shape errors
    assert lib.ppo_solve(p, p, 0, p, p, 1, 1, p, p, p, s) == binding.PPO_EINVAL
    assert lib.ppo_solve(p, p, 4, p, p, 5, 1, p, p, p, s) == binding.PPO_EINVAL
    assert lib.ppo_solve(p, p, 4, p, p, 0, 1, p, p, p, s) == binding.PPO_EINVAL
    assert lib.ppo_solve(p, p, 4, p, p, 2, -1, p, p, p, s) == binding.PPO_EINVAL
    assert lib.ppo_solve(p, p, 129, p, p, 2, 1, p, p, p, s) == binding.PPO_ETOOBIG
    assert lib.ppo_solve(p, p, 100, p, p, 13, 1, p, p, p, s) == binding.PPO_ETOOBIG
    # null pointers
    assert lib.ppo_solve(null, p, 4, p, p, 2, 1, p, p, p, s) == binding.PPO_EINVAL
    assert lib.ppo_solve(p, p, 4, p, p, 2, 1, null, p, p, s) == binding.PPO_EINVAL
    assert lib.ppo_solve(p, p, 4, p, p, 2, 1, p, null, p, s) == binding.PPO_EINVAL
    # empty batch is a successful no-op, even with null pointers
    assert lib.ppo_solve(null, null, 4, null, null, 2, 0, null, null, null, s) == binding.PPO_OK
    assert lib.ppo_init_keys(null, 0, s) == binding.PPO_OK
    assert lib.ppo_init_keys(null, 3, s) == binding.PPO_EINVAL
    # workspace too small / missing
    assert lib.ppo_solve_ws(p, p, 4, p, p, 2, 1, p, p, p, p, 16, s) == binding.PPO_ENOSPC
    assert lib.ppo_solve_ws(p, p, 4, p, p, 2, 1, p, p, p, null, 1 << 20, s) == binding.PPO_EINVAL
    # the entry point that allocates nothing: same shape checks, and a batch beyond its array is refused
    assert lib.ppo_solve_static(p, p, 4, p, p, 5, 1, p, p, p, s) == binding.PPO_EINVAL
    assert lib.ppo_solve_static(p, p, 100, p, p, 13, 1, p, p, p, s) == binding.PPO_ETOOBIG
    assert lib.ppo_solve_static(null, p, 4, p, p, 2, 1, p, p, p, s) == binding.PPO_EINVAL
    assert lib.ppo_solve_static(null, null, 4, null, null, 2, 0, null, null, null, s) == binding.PPO_OK
    assert binding.ppo_workspace_bytes(100, 10, 112) <= binding.PPO_STATIC_SCRATCH_BYTES < binding.ppo_workspace_bytes(100, 10, 113)
    assert lib.ppo_solve_static(p, p, 100, p, p, 10, 128, p, p, p, s) == binding.PPO_ENOSPC
    # rank ranges
    assert lib.ppo_solve_range(4, 3, 1, p, 1 << 20, 5, 4, p, s) == binding.PPO_EINVAL
    assert lib.ppo_solve_range(4, 3, 1, p, 1 << 20, 0, 7, p, s) == binding.PPO_EINVAL
    assert lib.ppo_solve_range(4, 3, 1, p, 16, 0, 6, p, s) == binding.PPO_ENOSPC
    assert lib.ppo_solve_range_bounded(4, 3, 1, p, 1 << 20, 5, 4, p, None, s) == binding.PPO_EINVAL
    assert lib.ppo_solve_range_bounded(4, 3, 1, p, 16, 0, 6, p, None, s) == binding.PPO_ENOSPC
    assert lib.ppo_prepare(p, p, 4, p, p, 3, 1, p, 16, s) == binding.PPO_ENOSPC
    assert lib.ppo_prepare(p, null, 4, p, p, 3, 1, p, 1 << 20, s) == binding.PPO_EINVAL
    assert lib.ppo_eval_orderings(p, p, 4, p, p, 3, 0, 7, p, s) == binding.PPO_EINVAL
    assert lib.ppo_eval_orderings(p, p, 4, p, p, 3, 2, 2, p, s) == binding.PPO_OK   # empty range
    assert lib.ppo_finalize(4, 2, 1, p, 1 << 20, null, p, p, p, s) == binding.PPO_EINVAL
    # misaligned workspace (256 bytes), keys and counters (8 bytes)
    odd_ws, odd_key = C.c_void_p(0x1010), C.c_void_p(0x1004)
    assert lib.ppo_prepare(p, p, 4, p, p, 3, 1, odd_ws, 1 << 20, s) == binding.PPO_EINVAL
    assert lib.ppo_solve_ws(p, p, 4, p, p, 2, 1, p, p, p, odd_ws, 1 << 20, s) == binding.PPO_EINVAL
    assert lib.ppo_solve_range(4, 3, 1, odd_ws, 1 << 20, 0, 6, p, s) == binding.PPO_EINVAL
    assert lib.ppo_solve_range(4, 3, 1, p, 1 << 20, 0, 6, odd_key, s) == binding.PPO_EINVAL
    assert lib.ppo_solve_range_bounded(4, 3, 1, p, 1 << 20, 0, 6, p, odd_key, s) == binding.PPO_EINVAL
    assert lib.ppo_solve_subsets(4, 3, 1, odd_ws, 1 << 20, p, s) == binding.PPO_EINVAL
    assert lib.ppo_finalize(4, 2, 1, p, 1 << 20, odd_key, p, p, p, s) == binding.PPO_EINVAL
    assert lib.ppo_init_keys(odd_key, 3, s) == binding.PPO_EINVAL


def test_cluster_entry_point_without_a_gpu(lib):
    p, null, s = C.c_void_p(0x1000), C.c_void_p(0), C.c_void_p(0)
    lib.ppo_cluster_workspace_bytes.restype = C.c_size_t
    one = lib.ppo_cluster_workspace_bytes(100, 20, 1)
    rows = 20 * (1 << 19) * 100 * 2                                     # n 2^(n-1) rows of L 16-bit entries
    assert rows <= one < rows + (1 << 20) and one % 256 == 0
    assert lib.ppo_cluster_workspace_bytes(100, 21, 1) == 0 and lib.ppo_cluster_workspace_bytes(129, 5, 1) == 0
    assert lib.ppo_cluster_workspace_bytes(100, 20, 64) < 64 * one      # rows capped, tables for all
    assert lib.ppo_cluster_workspace_bytes(4, 9, 3) > 0                 # more nodes than layers is allowed
    args = lambda L, n, ni, pmax, ws=p, nbytes=1 << 30: (p, p, L, p, p, n, ni, pmax, p, p, p, p, ws, nbytes, s)
    assert lib.ppo_solve_cluster(*args(0, 3, 1, 1)) == binding.PPO_EINVAL
    assert lib.ppo_solve_cluster(*args(10, 0, 1, 1)) == binding.PPO_EINVAL
    assert lib.ppo_solve_cluster(*args(10, 3, -1, 1)) == binding.PPO_EINVAL
    assert lib.ppo_solve_cluster(*args(10, 3, 1, 0)) == binding.PPO_EINVAL
    assert lib.ppo_solve_cluster(*args(10, 3, 1, 4)) == binding.PPO_EINVAL
    assert lib.ppo_solve_cluster(*args(10, 21, 1, 2)) == binding.PPO_ETOOBIG
    assert lib.ppo_solve_cluster(*args(129, 3, 1, 2)) == binding.PPO_ETOOBIG
    assert lib.ppo_solve_cluster(*args(10, 3, 0, 2, null, 0)) == binding.PPO_OK
    assert lib.ppo_solve_cluster(*args(10, 3, 1, 2, null)) == binding.PPO_EINVAL
    assert lib.ppo_solve_cluster(*args(10, 3, 1, 2, C.c_void_p(0x1010))) == binding.PPO_EINVAL
    assert lib.ppo_solve_cluster(*args(10, 3, 1, 2, p, 64)) == binding.PPO_ENOSPC
    assert lib.ppo_solve_cluster(p, p, 10, p, p, 3, 1, 2, null, p, p, p, p, 1 << 30, s) == binding.PPO_EINVAL


def test_cluster_few_refuses_bad_arguments(lib):
    p, null, s = C.c_void_p(0x1000), C.c_void_p(0), C.c_void_p(0)

    def args(L, n, n_inst, pmax, ws=p, size=1 << 40):
        return (p, p, L, p, p, n, n_inst, pmax, p, p, p, p, ws, size, s)

    f = lib.ppo_solve_cluster_few
    assert f(*args(0, 3, 1, 2)) == binding.PPO_EINVAL
    assert f(*args(10, 0, 1, 1)) == binding.PPO_EINVAL
    assert f(*args(10, 3, 1, 0)) == binding.PPO_EINVAL
    assert f(*args(10, 3, 1, 4)) == binding.PPO_EINVAL
    assert f(*args(10, 3, -1, 2)) == binding.PPO_EINVAL
    assert f(*args(10, 65, 1, 2)) == binding.PPO_ETOOBIG
    assert f(*args(129, 3, 1, 2)) == binding.PPO_ETOOBIG
    assert f(*args(100, 30, 1, 9)) == binding.PPO_ETOOBIG
    assert f(*args(100, 64, 1, 8)) == binding.PPO_ETOOBIG      # more than 2^31 rows
    assert f(*args(5, 30, 1, 9, p, 64)) == binding.PPO_ENOSPC  # at most L = 5 segments: a legal shape
    assert f(*args(10, 3, 0, 2, null, 0)) == binding.PPO_OK
    assert f(*args(10, 3, 1, 2, null)) == binding.PPO_EINVAL
    assert f(*args(10, 3, 1, 2, C.c_void_p(0x1010))) == binding.PPO_EINVAL
    assert f(*args(10, 3, 1, 2, p, 64)) == binding.PPO_ENOSPC
    assert f(p, p, 10, p, p, 3, 1, 2, null, p, p, p, p, 1 << 30, s) == binding.PPO_EINVAL
    assert lib.ppo_cluster_few_workspace_bytes(100, 50, 5, 1) > 0
    assert lib.ppo_cluster_few_workspace_bytes(100, 64, 8, 1) == 0


def test_partition_and_front_end_refuse_bad_arguments(lib):
    p, null, s = C.c_void_p(0x1000), C.c_void_p(0), C.c_void_p(0)
    assert lib.ppo_min_sum_partition(p, p, 0, p, 1, p, p, p, s) == binding.PPO_EINVAL
    assert lib.ppo_min_sum_partition(p, p, 129, p, 1, p, p, p, s) == binding.PPO_ETOOBIG
    assert lib.ppo_min_sum_partition(p, p, 10, p, -1, p, p, p, s) == binding.PPO_EINVAL
    assert lib.ppo_min_sum_partition(p, p, 10, p, 0, null, null, null, s) == binding.PPO_OK
    assert lib.ppo_min_sum_partition(p, p, 10, null, 1, p, p, p, s) == binding.PPO_EINVAL
    assert lib.ppo_min_sum_partition(p, p, 10, p, 1, p, null, p, s) == binding.PPO_EINVAL
    assert lib.ppo_probe_valu(0, 10, p, s) == binding.PPO_EINVAL
    assert lib.ppo_probe_valu(5, 10, p, s) == binding.PPO_EINVAL
    assert lib.ppo_probe_valu(2, 0, p, s) == binding.PPO_EINVAL
    assert lib.ppo_probe_valu(2, 10, null, s) == binding.PPO_EINVAL
    assert lib.ppo_min_sum_partition(p, p, 10, p, 1, p, p, C.c_void_p(0x1004), s) == binding.PPO_EINVAL
    assert lib.ppo_chain_from_dag(0, 0, null, null, p, p, 4, p, p, p, p) == binding.PPO_EINVAL
    assert lib.ppo_chain_from_dag(3, 2, null, p, p, p, 4, p, p, p, p) == binding.PPO_EINVAL
