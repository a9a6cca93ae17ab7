"""ctypes access to the CPU oracle of the search with the compute-time term (oracle/ppo_ct_oracle.c; Sec. I, Eq. 1).

TEST INFRASTRUCTURE ONLY.  Tests, the smoke check and the benchmark's CPU-baseline leg may import this; the
product package never does.  It shares no code with the HIP library and takes host (numpy) arrays only.
Every function takes ONE instance: t, m, w [L]; M, v [k]; B [k, k].
"""
from __future__ import annotations

import ctypes as C
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ppo_ct_oracle.c")
_LIB = os.path.join(_HERE, "libppo_ct_oracle.so")
# The mutation tests point this at an altered copy of the source; the library is then built beside that copy.
if os.environ.get("PPO_CT_ORACLE_SOURCE"):
    _SRC = os.path.abspath(os.environ["PPO_CT_ORACLE_SOURCE"])
    _LIB = os.path.join(os.path.dirname(_SRC), "libppo_ct_oracle_mutant.so")


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"compute-term oracle error {code}")
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
        fp, ip, u64 = C.POINTER(C.c_float), C.POINTER(C.c_int32), C.c_uint64
        inst = [fp, fp, fp, C.c_int, fp, fp, fp, C.c_int]
        _lib.ppo_ct_oracle_bruteforce.argtypes = inst + [fp, ip, ip]
        _lib.ppo_ct_oracle_subset_dp.argtypes = inst + [fp, ip, ip]
        _lib.ppo_ct_oracle_exhaustive.argtypes = inst + [u64, u64, fp, fp, ip, ip]
        _lib.ppo_ct_oracle_evaluate.argtypes = inst + [ip, ip, fp, ip]
    return _lib


def _inst(t, m, w, M, v, B):
    t, m, w, M, v, B = (np.ascontiguousarray(x, dtype=np.float32) for x in (t, m, w, M, v, B))
    L, k = t.shape[0], M.shape[0]
    assert t.shape == m.shape == w.shape == (L,) and M.shape == v.shape == (k,) and B.shape == (k, k)
    fp = lambda a: a.ctypes.data_as(C.POINTER(C.c_float))
    return (t, m, w, M, v, B), [fp(t), fp(m), fp(w), L, fp(M), fp(v), fp(B), k], L, k


def _ip(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _solve(fn, t, m, w, M, v, B, extra=()):
    keep, args, L, k = _inst(t, m, w, M, v, B)
    beta = C.c_float()
    cuts = np.full(max(k - 1, 1), -1, np.int32)
    order = np.full(k, -1, np.int32)
    rc = fn(*args, *extra, C.byref(beta), _ip(cuts), _ip(order))
    if rc != 0:
        raise OracleError(rc)
    return np.float32(beta.value), cuts[: k - 1].copy(), order


def bruteforce(t, m, w, M, v, B):
    """(beta, cuts [k-1], order [k]) from the definition: every cut vector with every permutation."""
    return _solve(lib().ppo_ct_oracle_bruteforce, t, m, w, M, v, B)


def subset_dp(t, m, w, M, v, B):
    """The same from a dynamic programme over node subsets."""
    return _solve(lib().ppo_ct_oracle_subset_dp, t, m, w, M, v, B)


def exhaustive(t, m, w, M, v, B, rank_range=None):
    """The same from one chain DP per ordering (those with rank in rank_range, default all)."""
    k = np.asarray(M).shape[0]
    r0, r1 = rank_range if rank_range is not None else (0, math.factorial(k))
    return _solve(lib().ppo_ct_oracle_exhaustive, t, m, w, M, v, B, (int(r0), int(r1), None))


def eval_orderings(t, m, w, M, v, B, rank_begin, rank_end):
    """beta of every ordering with rank in [rank_begin, rank_end)."""
    keep, args, L, k = _inst(t, m, w, M, v, B)
    out = np.empty(int(rank_end - rank_begin), np.float32)
    rc = lib().ppo_ct_oracle_exhaustive(*args, int(rank_begin), int(rank_end), out.ctypes.data_as(C.POINTER(C.c_float)),
                                        None, None, None)
    if rc != 0:
        raise OracleError(rc)
    return out


def evaluate(t, m, w, M, v, B, order, cuts):
    """(beta, feasible) of one explicit solution, from the definition."""
    keep, args, L, k = _inst(t, m, w, M, v, B)
    o = np.ascontiguousarray(order, dtype=np.int32)
    c = np.ascontiguousarray(cuts, dtype=np.int32) if k > 1 else np.zeros(1, np.int32)
    beta, feas = C.c_float(), C.c_int32()
    rc = lib().ppo_ct_oracle_evaluate(*args, _ip(o), _ip(c), C.byref(beta), C.byref(feas))
    if rc != 0:
        raise OracleError(rc)
    return np.float32(beta.value), bool(feas.value)
