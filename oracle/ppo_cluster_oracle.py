"""ctypes access to the CPU oracle of the cluster form (oracle/ppo_cluster_oracle.c).

TEST INFRASTRUCTURE ONLY.  Tests, the smoke check and the benchmark's CPU-baseline leg may import
this; the product package never does.  It shares no code with the HIP library and takes host
(numpy) arrays only.  Every function takes ONE instance: t, m [L]; M [n]; B [n, n].
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ppo_cluster_oracle.c")
_LIB = os.path.join(_HERE, "libppo_cluster_oracle.so")
# The mutation tests (tests/test_oracle_mutants.py) point this at an altered copy of the source to show that the
# pins notice; the library is then built beside that copy.
if os.environ.get("PPO_CLUSTER_ORACLE_SOURCE"):
    _SRC = os.path.abspath(os.environ["PPO_CLUSTER_ORACLE_SOURCE"])
    _LIB = os.path.join(os.path.dirname(_SRC), "libppo_cluster_oracle_mutant.so")

ERRORS = {0: "ok", -1: "invalid argument", -2: "too big", -3: "data precondition violated", -4: "out of memory"}


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"cluster oracle error {code}: {ERRORS.get(code, '?')}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
                               "-Wall", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        fp, ip = C.POINTER(C.c_float), C.POINTER(C.c_int32)
        inst = [fp, fp, C.c_int, fp, fp, C.c_int]
        out = [fp, ip, ip, ip]
        _lib.ppo_cluster_oracle_bruteforce.argtypes = inst + [C.c_int] + out
        _lib.ppo_cluster_oracle_exhaustive.argtypes = inst + [C.c_int] + out + [C.POINTER(C.c_uint64)]
        _lib.ppo_cluster_oracle_subset_dp.argtypes = inst + [C.c_int] + out
        _lib.ppo_cluster_oracle_sequence.argtypes = inst + [ip, C.c_int, fp]
    return _lib


def _inst(t, m, M, B):
    t, m, M, B = (np.ascontiguousarray(x, dtype=np.float32) for x in (t, m, M, B))
    L, n = t.shape[0], M.shape[0]
    assert t.shape == (L,) and m.shape == (L,) and M.shape == (n,) and B.shape == (n, n)
    fp = lambda a: a.ctypes.data_as(C.POINTER(C.c_float))
    return (t, m, M, B), [fp(t), fp(m), L, fp(M), fp(B), n], L, n


def _solve(fn, t, m, M, B, max_segments, extra=()):
    keep, args, L, n = _inst(t, m, M, B)
    pmax = n if max_segments is None else int(max_segments)
    beta, segs = C.c_float(), C.c_int32()
    cuts = np.full(max(n - 1, 1), -1, np.int32)
    order = np.full(n, -1, np.int32)
    ip = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    rc = fn(*args, pmax, C.byref(beta), C.byref(segs), ip(cuts), ip(order), *extra)
    if rc != 0:
        raise OracleError(rc)
    return np.float32(beta.value), int(segs.value), cuts[: n - 1].copy(), order


def bruteforce(t, m, M, B, max_segments=None):
    """(beta, segments, cuts [n-1], order [n]) from the definition: every node sequence, every cut vector."""
    return _solve(lib().ppo_cluster_oracle_bruteforce, t, m, M, B, max_segments)


def exhaustive(t, m, M, B, max_segments=None):
    """The same from one chain DP per node sequence."""
    visited = C.c_uint64(0)
    return _solve(lib().ppo_cluster_oracle_exhaustive, t, m, M, B, max_segments, (C.byref(visited),))


def subset_dp(t, m, M, B, max_segments=None):
    """The same from a dynamic programme over sets of unused nodes."""
    return _solve(lib().ppo_cluster_oracle_subset_dp, t, m, M, B, max_segments)


def sequence_beta(t, m, M, B, seq) -> np.float32:
    """Least bottleneck of ONE node sequence over its cut vectors (+inf if none is feasible)."""
    keep, args, L, n = _inst(t, m, M, B)
    s = np.ascontiguousarray(seq, dtype=np.int32)
    beta = C.c_float()
    rc = lib().ppo_cluster_oracle_sequence(*args, s.ctypes.data_as(C.POINTER(C.c_int32)), len(s), C.byref(beta))
    if rc != 0:
        raise OracleError(rc)
    return np.float32(beta.value)
