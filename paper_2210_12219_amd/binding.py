"""Thin ctypes binding over the C ABI of libppo.so (include/ppo.h), same names as the C entry points.

Argument marshalling only: every step of the search runs in the HIP kernels.  PyTorch supplies
device memory and the current stream.  There is no CPU fallback: if the library is missing or
no GPU is present, calls fail loudly.
"""
from __future__ import annotations

import ctypes as C
import math
import os

PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG, "libppo.so")

PPO_OK, PPO_EINVAL, PPO_ETOOBIG, PPO_EHIP, PPO_ENOSPC = 0, -1, -2, -3, -4
PPO_MAX_K, PPO_MAX_L = 12, 128
PPO_CLUSTER_MAX_N = 20
PPO_CLUSTER_FEW_MAX_N, PPO_CLUSTER_FEW_MAX_SEGMENTS = 64, 8
PPO_KEY_NONE = 0xFFFFFFFFFFFFFFFF


class PpoError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"ppo error {code}: {text}")
        self.code = code


_lib = None


def load() -> C.CDLL:
    """Load libppo.so (built by paper_2210_12219_amd.build); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2210_12219_amd.build` first")
        # PyTorch ships its own HIP runtime; it has to be in the process before libppo.so is, so that both
        # use the same one (tensors' device pointers mean nothing to a second runtime).
        import torch  # noqa: F401
        lib = C.CDLL(LIB_PATH)
        vp, i, u64, sz = C.c_void_p, C.c_int, C.c_uint64, C.c_size_t
        inst = [vp, vp, i, vp, vp, i]
        lib.ppo_version.argtypes = []
        lib.ppo_strerror.argtypes = [i]
        lib.ppo_strerror.restype = C.c_char_p
        lib.ppo_set_enumeration.argtypes = [i]
        lib.ppo_workspace_bytes.argtypes = [i, i, i]
        lib.ppo_workspace_bytes.restype = sz
        lib.ppo_solve.argtypes = inst + [i, vp, vp, vp, vp]
        lib.ppo_solve_static.argtypes = inst + [i, vp, vp, vp, vp]
        lib.ppo_solve_ws.argtypes = inst + [i, vp, vp, vp, vp, sz, vp]
        lib.ppo_prepare.argtypes = inst + [i, vp, sz, vp]
        lib.ppo_init_keys.argtypes = [vp, i, vp]
        lib.ppo_solve_range.argtypes = [i, i, i, vp, sz, u64, u64, vp, vp]
        lib.ppo_solve_range_bounded.argtypes = [i, i, i, vp, sz, u64, u64, vp, vp, vp]
        lib.ppo_solve_subsets.argtypes = [i, i, i, vp, sz, vp, vp]
        lib.ppo_finalize.argtypes = [i, i, i, vp, sz, vp, vp, vp, vp, vp]
        lib.ppo_eval_orderings.argtypes = inst + [u64, u64, vp, vp]
        inst_ct = [vp, vp, vp, i, vp, vp, vp, i]
        lib.ppo_solve_ct.argtypes = inst_ct + [i, vp, vp, vp, vp]
        lib.ppo_eval_orderings_ct.argtypes = inst_ct + [u64, u64, vp, vp]
        lib.ppo_chain_from_dag.argtypes = [i, i, vp, vp, vp, vp, i, vp, vp, vp, vp]
        lib.ppo_min_sum_partition.argtypes = [vp, vp, i, vp, i, vp, vp, vp, vp]
        lib.ppo_place_kpath.argtypes = [vp, vp, i, vp, vp, i, i, i, vp, vp, vp, vp, vp, vp]
        lib.ppo_place_baseline.argtypes = [vp, vp, i, vp, vp, i, i, i, vp, i, vp, vp, vp, vp, vp]
        lib.ppo_cluster_workspace_bytes.argtypes = [i, i, i]
        lib.ppo_cluster_workspace_bytes.restype = sz
        lib.ppo_solve_cluster.argtypes = inst + [i, i, vp, vp, vp, vp, vp, sz, vp]
        lib.ppo_cluster_few_workspace_bytes.argtypes = [i, i, i, i]
        lib.ppo_cluster_few_workspace_bytes.restype = sz
        lib.ppo_solve_cluster_few.argtypes = inst + [i, i, vp, vp, vp, vp, vp, sz, vp]
        lib.ppo_probe_valu.argtypes = [i, i, vp, vp]
        _lib = lib
    return _lib


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("ppo needs a GPU: torch.cuda.is_available() is False")
    return torch


def _check(rc: int):
    if rc != PPO_OK:
        raise PpoError(rc, load().ppo_strerror(rc).decode())


def _stream(stream):
    torch = _torch()
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _dev(x, dtype):
    torch = _torch()
    assert x.is_cuda and x.dtype == dtype and x.is_contiguous(), "expected a contiguous device tensor"
    return C.c_void_p(x.data_ptr())


def _shape(t, m, M, B):
    n, L = t.shape
    k = M.shape[1]
    assert tuple(m.shape) == (n, L) and tuple(M.shape) == (n, k) and tuple(B.shape) == (n, k, k)
    return n, L, k


def ppo_version() -> int:
    return load().ppo_version()


def ppo_strerror(code: int) -> str:
    return load().ppo_strerror(code).decode()


PPO_ENUM_AUTO, PPO_ENUM_GENERIC, PPO_ENUM_GROUPED = 0, 1, 2


def ppo_set_enumeration(variant: int):
    _check(load().ppo_set_enumeration(variant))


def ppo_workspace_bytes(L: int, k: int, n_inst: int) -> int:
    return int(load().ppo_workspace_bytes(L, k, n_inst))


def to_device(w, device="cuda:0"):
    """Copy a workloads.Workload's arrays to the GPU; returns (t, m, M, B) float32 tensors."""
    torch = _torch()
    return tuple(torch.from_numpy(a).to(device) for a in (w.t, w.m, w.M, w.B))


def alloc_outputs(n_inst: int, k: int, device="cuda:0"):
    torch = _torch()
    return (torch.empty(n_inst, dtype=torch.float32, device=device),
            torch.empty((n_inst, max(k - 1, 0)), dtype=torch.int32, device=device),
            torch.empty((n_inst, k), dtype=torch.int32, device=device))


def ppo_solve(t, m, M, B, out=None, workspace=None, stream=None):
    """beta [n], cuts [n,k-1], order [n,k] for device tensors t,m [n,L], M [n,k], B [n,k,k].
    Enqueues on the stream and returns without synchronising."""
    torch = _torch()
    n, L, k = _shape(t, m, M, B)
    beta, cuts, order = out if out is not None else alloc_outputs(n, k, t.device)
    f32, i32 = torch.float32, torch.int32
    args = [_dev(t, f32), _dev(m, f32), L, _dev(M, f32), _dev(B, f32), k, n, _dev(beta, f32),
            C.c_void_p(cuts.data_ptr()), _dev(order, i32)]
    if workspace is None:
        _check(load().ppo_solve(*args, _stream(stream)))
    else:
        assert workspace.is_cuda and workspace.dtype == torch.uint8
        _check(load().ppo_solve_ws(*args, C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream(stream)))
    return beta, cuts, order


PPO_STATIC_SCRATCH_BYTES = 16 << 20


def ppo_solve_static(t, m, M, B, out, stream=None):
    """ppo_solve with the library's own static scratch: allocates nothing (the caller brings the outputs)."""
    torch = _torch()
    n, L, k = _shape(t, m, M, B)
    beta, cuts, order = out
    f32, i32 = torch.float32, torch.int32
    _check(load().ppo_solve_static(_dev(t, f32), _dev(m, f32), L, _dev(M, f32), _dev(B, f32), k, n, _dev(beta, f32),
                                   C.c_void_p(cuts.data_ptr()), _dev(order, i32), _stream(stream)))
    return beta, cuts, order


def alloc_workspace(L: int, k: int, n_inst: int, device="cuda:0"):
    torch = _torch()
    return torch.empty(max(ppo_workspace_bytes(L, k, n_inst), 1), dtype=torch.uint8, device=device)


def ppo_prepare(t, m, M, B, workspace, stream=None):
    """Stage 1: per-instance tables into workspace (uint8 device tensor)."""
    torch = _torch()
    n, L, k = _shape(t, m, M, B)
    f32 = torch.float32
    assert workspace.is_cuda and workspace.dtype == torch.uint8
    _check(load().ppo_prepare(_dev(t, f32), _dev(m, f32), L, _dev(M, f32), _dev(B, f32), k, n,
                              C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream(stream)))


def ppo_init_keys(best_key, stream=None):
    torch = _torch()
    assert best_key.dtype == torch.int64 and best_key.is_cuda
    _check(load().ppo_init_keys(C.c_void_p(best_key.data_ptr()), best_key.numel(), _stream(stream)))


def ppo_solve_range(L, k, n_inst, workspace, rank_begin, rank_end, best_key, stream=None):
    """Stage 2: fold the orderings with rank in [rank_begin, rank_end) into best_key (int64 tensor
    holding the unsigned 64-bit keys)."""
    torch = _torch()
    assert best_key.dtype == torch.int64 and best_key.numel() == n_inst and workspace.dtype == torch.uint8
    _check(load().ppo_solve_range(L, k, n_inst, C.c_void_p(workspace.data_ptr()), workspace.numel(), int(rank_begin),
                                  int(rank_end), C.c_void_p(best_key.data_ptr()), _stream(stream)))


def ppo_solve_range_bounded(L, k, n_inst, workspace, rank_begin, rank_end, best_key, skipped_groups=None, stream=None):
    """Stage 2 with shared prefix rows and skipped groups: same best_key as ppo_solve_range.  skipped_groups
    (int64 tensor [n_inst], zeroed by the caller) counts the groups of 360 orderings skipped per instance."""
    torch = _torch()
    assert best_key.dtype == torch.int64 and best_key.numel() == n_inst and workspace.dtype == torch.uint8
    assert skipped_groups is None or (skipped_groups.dtype == torch.int64 and skipped_groups.numel() == n_inst)
    sk = C.c_void_p(skipped_groups.data_ptr()) if skipped_groups is not None else None
    _check(load().ppo_solve_range_bounded(L, k, n_inst, C.c_void_p(workspace.data_ptr()), workspace.numel(),
                                          int(rank_begin), int(rank_end), C.c_void_p(best_key.data_ptr()), sk,
                                          _stream(stream)))


def ppo_solve_subsets(L, k, n_inst, workspace, best_key, stream=None):
    """Stage 2 by dynamic programming over node subsets: best_key as after ppo_solve_range over [0, k!)."""
    torch = _torch()
    assert best_key.dtype == torch.int64 and best_key.numel() == n_inst and workspace.dtype == torch.uint8
    _check(load().ppo_solve_subsets(L, k, n_inst, C.c_void_p(workspace.data_ptr()), workspace.numel(),
                                    C.c_void_p(best_key.data_ptr()), _stream(stream)))


def ppo_finalize(L, k, n_inst, workspace, best_key, out=None, stream=None):
    """Stage 3: (beta, cuts, order) from best_key."""
    torch = _torch()
    beta, cuts, order = out if out is not None else alloc_outputs(n_inst, k, workspace.device)
    f32, i32 = torch.float32, torch.int32
    _check(load().ppo_finalize(L, k, n_inst, C.c_void_p(workspace.data_ptr()), workspace.numel(),
                               C.c_void_p(best_key.data_ptr()), _dev(beta, f32), C.c_void_p(cuts.data_ptr()),
                               _dev(order, i32), _stream(stream)))
    return beta, cuts, order


def ppo_eval_orderings(t, m, M, B, rank_begin, rank_end, stream=None):
    """beta of every ordering of ONE instance (t,m [L]; M [k]; B [k,k]) with rank in the range."""
    torch = _torch()
    L, k = t.shape[0], M.shape[0]
    f32 = torch.float32
    out = torch.empty(int(rank_end - rank_begin), dtype=f32, device=t.device)
    _check(load().ppo_eval_orderings(_dev(t, f32), _dev(m, f32), L, _dev(M, f32), _dev(B, f32), k, int(rank_begin),
                                     int(rank_end), C.c_void_p(out.data_ptr()), _stream(stream)))
    return out


def ppo_solve_ct(t, m, w, M, v, B, out=None, stream=None):
    """The search with the compute-time term: w [n,L] per-layer work, v [n,k] node speeds; (beta, cuts, order)."""
    torch = _torch()
    n, L, k = _shape(t, m, M, B)
    assert tuple(w.shape) == (n, L) and tuple(v.shape) == (n, k)
    beta, cuts, order = out if out is not None else alloc_outputs(n, k, t.device)
    f32, i32 = torch.float32, torch.int32
    _check(load().ppo_solve_ct(_dev(t, f32), _dev(m, f32), _dev(w, f32), L, _dev(M, f32), _dev(v, f32), _dev(B, f32), k, n,
                               _dev(beta, f32), C.c_void_p(cuts.data_ptr()), _dev(order, i32), _stream(stream)))
    return beta, cuts, order


def ppo_eval_orderings_ct(t, m, w, M, v, B, rank_begin, rank_end, stream=None):
    """beta (with the compute-time term) of every ordering of ONE instance with rank in the range."""
    torch = _torch()
    L, k = t.shape[0], M.shape[0]
    f32 = torch.float32
    out = torch.empty(int(rank_end - rank_begin), dtype=f32, device=t.device)
    _check(load().ppo_eval_orderings_ct(_dev(t, f32), _dev(m, f32), _dev(w, f32), L, _dev(M, f32), _dev(v, f32),
                                        _dev(B, f32), k, int(rank_begin), int(rank_end), C.c_void_p(out.data_ptr()),
                                        _stream(stream)))
    return out


def ppo_min_sum_partition(t, m, kappa, stream=None):
    """The paper's partitioning step (least sum of transfer sizes): (segs [n], cuts [n, L-1], sum [n] float64)."""
    torch = _torch()
    n_inst, L = t.shape
    f32 = torch.float32
    segs = torch.empty(n_inst, dtype=torch.int32, device=t.device)
    cuts = torch.empty((n_inst, max(L - 1, 0)), dtype=torch.int32, device=t.device)
    total = torch.empty(n_inst, dtype=torch.float64, device=t.device)
    _check(load().ppo_min_sum_partition(_dev(t, f32), _dev(m, f32), L, _dev(kappa, f32), n_inst,
                                        C.c_void_p(segs.data_ptr()), C.c_void_p(cuts.data_ptr()),
                                        C.c_void_p(total.data_ptr()), _stream(stream)))
    return segs, cuts, total


PPO_BASELINE_JOINT, PPO_BASELINE_RANDOM = 1, 2
PPO_HEURISTIC_MAX_N = 64


def _place_outputs(torch, n_inst, L, n, device):
    return (torch.empty(n_inst, dtype=torch.float32, device=device), torch.empty(n_inst, dtype=torch.int32, device=device),
            torch.empty((n_inst, max(L - 1, 0)), dtype=torch.int32, device=device),
            torch.empty((n_inst, n), dtype=torch.int32, device=device))


def ppo_place_kpath(t, m, kappa, B, n_classes, stream=None):
    """The paper's placement algorithm: (beta [n], segs [n], cuts [n, L-1], order [n, nodes], classes used [n])."""
    torch = _torch()
    n_inst, L = t.shape
    n = B.shape[1]
    f32, i32 = torch.float32, torch.int32
    beta, segs, cuts, order = _place_outputs(torch, n_inst, L, n, t.device)
    used = torch.empty(n_inst, dtype=i32, device=t.device)
    _check(load().ppo_place_kpath(_dev(t, f32), _dev(m, f32), L, _dev(kappa, f32), _dev(B, f32), n, n_inst, int(n_classes),
                                  _dev(beta, f32), _dev(segs, i32), C.c_void_p(cuts.data_ptr()), _dev(order, i32),
                                  _dev(used, i32), _stream(stream)))
    return beta, segs, cuts, order, used


def ppo_place_baseline(t, m, kappa, B, kind, draws=None, stream=None):
    """The paper's comparison systems: (beta, segs, cuts, order); draws [n, n_draws] for the random one."""
    torch = _torch()
    n_inst, L = t.shape
    n = B.shape[1]
    f32, i32 = torch.float32, torch.int32
    beta, segs, cuts, order = _place_outputs(torch, n_inst, L, n, t.device)
    n_draws = 0 if draws is None else draws.shape[1]
    _check(load().ppo_place_baseline(_dev(t, f32), _dev(m, f32), L, _dev(kappa, f32), _dev(B, f32), n, n_inst, int(kind),
                                     None if draws is None else _dev(draws, f32), n_draws, _dev(beta, f32), _dev(segs, i32),
                                     C.c_void_p(cuts.data_ptr()), _dev(order, i32), _stream(stream)))
    return beta, segs, cuts, order


def ppo_chain_from_dag(n_vertices, edges, weight, out_size):
    """Host routine: (t [L], m [L], point [L]) of the chain of a layer graph; edges is a sequence of (src, dst)."""
    import numpy as np
    e = np.ascontiguousarray(np.asarray(edges, dtype=np.int32).reshape(-1, 2))
    src, dst = np.ascontiguousarray(e[:, 0]), np.ascontiguousarray(e[:, 1])
    w = np.ascontiguousarray(weight, dtype=np.float32)
    o = np.ascontiguousarray(out_size, dtype=np.float32)
    assert w.shape == (n_vertices,) and o.shape == (n_vertices,)
    cap = n_vertices + 1
    t, m = np.zeros(cap, np.float32), np.zeros(cap, np.float32)
    point, L = np.zeros(cap, np.int32), C.c_int32(0)
    ptr = lambda a: C.c_void_p(a.ctypes.data)
    _check(load().ppo_chain_from_dag(n_vertices, len(src), ptr(src), ptr(dst), ptr(w), ptr(o), cap, ptr(t), ptr(m),
                                     ptr(point), C.cast(C.byref(L), C.c_void_p)))
    return t[:L.value].copy(), m[:L.value].copy(), point[:L.value].copy()


def ppo_cluster_workspace_bytes(L: int, n: int, n_inst: int) -> int:
    return int(load().ppo_cluster_workspace_bytes(L, n, n_inst))


def ppo_solve_cluster(t, m, M, B, max_segments=None, workspace=None, out=None, stream=None):
    """Cluster form: (beta [n_inst], segs [n_inst], cuts [n_inst, n-1], order [n_inst, n]) over every number of
    segments up to max_segments (default n) and every sequence of distinct nodes."""
    torch = _torch()
    n_inst, L = t.shape
    n = M.shape[1]
    f32, i32 = torch.float32, torch.int32
    if workspace is None:
        workspace = torch.empty(ppo_cluster_workspace_bytes(L, n, n_inst), dtype=torch.uint8, device=t.device)
    if out is None:
        out = (torch.empty(n_inst, dtype=f32, device=t.device), torch.empty(n_inst, dtype=i32, device=t.device),
               torch.empty((n_inst, max(n - 1, 0)), dtype=i32, device=t.device),
               torch.empty((n_inst, n), dtype=i32, device=t.device))
    beta, segs, cuts, order = out
    _check(load().ppo_solve_cluster(_dev(t, f32), _dev(m, f32), L, _dev(M, f32), _dev(B, f32), n, n_inst,
                                    n if max_segments is None else int(max_segments), _dev(beta, f32),
                                    _dev(segs, i32), C.c_void_p(cuts.data_ptr()), _dev(order, i32),
                                    C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream(stream)))
    return beta, segs, cuts, order


def ppo_cluster_few_workspace_bytes(L, n, max_segments, n_inst) -> int:
    return int(load().ppo_cluster_few_workspace_bytes(L, n, max_segments, n_inst))


def ppo_solve_cluster_few(t, m, M, B, max_segments, workspace=None, out=None, stream=None):
    """Cluster form for large clusters and few segments (n <= 64, max_segments <= 8): outputs as ppo_solve_cluster."""
    torch = _torch()
    n_inst, L = t.shape
    n = M.shape[1]
    f32, i32 = torch.float32, torch.int32
    if workspace is None:
        size = ppo_cluster_few_workspace_bytes(L, n, int(max_segments), n_inst)
        workspace = torch.empty(max(size, 256), dtype=torch.uint8, device=t.device)   # a bad shape is the call's to refuse
    if out is None:
        out = (torch.empty(n_inst, dtype=f32, device=t.device), torch.empty(n_inst, dtype=i32, device=t.device),
               torch.empty((n_inst, max(n - 1, 0)), dtype=i32, device=t.device),
               torch.empty((n_inst, n), dtype=i32, device=t.device))
    beta, segs, cuts, order = out
    _check(load().ppo_solve_cluster_few(_dev(t, f32), _dev(m, f32), L, _dev(M, f32), _dev(B, f32), n, n_inst,
                                        int(max_segments), _dev(beta, f32), _dev(segs, i32), C.c_void_p(cuts.data_ptr()),
                                        _dev(order, i32), C.c_void_p(workspace.data_ptr()), workspace.numel(),
                                        _stream(stream)))
    return beta, segs, cuts, order


def orderings_per_instance(k: int) -> int:
    return math.factorial(k)


def ppo_probe_valu(waves_per_simd, iters, sink=None, stream=None):
    """Enqueue the vector-ALU issue probe (a measurement aid); returns the sink tensor."""
    torch = _torch()
    if sink is None:
        sink = torch.empty(256 * 256 * waves_per_simd, dtype=torch.int32, device="cuda:0")
    _check(load().ppo_probe_valu(waves_per_simd, iters, sink.data_ptr(), _stream(stream)))
    return sink
