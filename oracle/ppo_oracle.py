"""ctypes access to the CPU oracle (oracle/ppo_oracle.c).

TEST INFRASTRUCTURE ONLY.  Tests, the smoke check and the benchmark's CPU-baseline
leg may import this; the product package never does.  It shares no code with the
HIP library and takes host (numpy) arrays only.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ppo_oracle.c")
_LIB = os.path.join(_HERE, "libppo_oracle.so")
# The mutation tests (tests/test_oracle_mutants.py) point this at an altered copy of the source to show that the
# pins notice; the library is then built beside that copy.
if os.environ.get("PPO_ORACLE_SOURCE"):
    _SRC = os.path.abspath(os.environ["PPO_ORACLE_SOURCE"])
    _LIB = os.path.join(os.path.dirname(_SRC), "libppo_oracle_mutant.so")

ERRORS = {0: "ok", -1: "invalid argument", -2: "too big", -3: "data precondition violated", -4: "out of memory"}


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle error {code}: {ERRORS.get(code, '?')}")
        self.code = code


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
                               "-Wall", "-o", tmp, _SRC, "-lpthread", "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        fp, ip = C.POINTER(C.c_float), C.POINTER(C.c_int32)
        u64p = C.POINTER(C.c_uint64)
        inst = [fp, fp, C.c_int, fp, fp, C.c_int]
        _lib.ppo_oracle_check_inputs.argtypes = inst + [C.c_int]
        _lib.ppo_oracle_rank.argtypes = [ip, C.c_int]
        _lib.ppo_oracle_rank.restype = C.c_uint64
        _lib.ppo_oracle_unrank.argtypes = [C.c_uint64, C.c_int, ip]
        _lib.ppo_oracle_unrank.restype = None
        _lib.ppo_oracle_evaluate.argtypes = inst + [ip, ip, fp, ip]
        _lib.ppo_oracle_bruteforce.argtypes = inst + [fp, ip, ip]
        _lib.ppo_oracle_exhaustive.argtypes = inst + [C.c_int, fp, ip, ip, C.c_int, u64p]
        _lib.ppo_oracle_exhaustive_range.argtypes = inst + [C.c_int, C.c_uint64, C.c_uint64, fp, ip, ip, C.c_int, u64p]
        _lib.ppo_oracle_eval_orderings.argtypes = inst + [C.c_uint64, C.c_uint64, fp, C.c_int, u64p]
        _lib.ppo_oracle_subset_dp.argtypes = inst + [C.c_int, fp, ip, ip, C.c_int]
    return _lib


def _f(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(C.POINTER(C.c_float))


def _i(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _batch(t, m, M, B):
    t, m, M, B = (np.ascontiguousarray(x, dtype=np.float32) for x in (t, m, M, B))
    if t.ndim == 1:
        t, m, M, B = t[None], m[None], M[None], B[None]
    n, L = t.shape
    k = M.shape[1]
    assert m.shape == (n, L) and M.shape == (n, k) and B.shape == (n, k, k)
    return t, m, M, B, n, L, k


def _check(rc):
    if rc != 0:
        raise OracleError(rc)


def default_threads() -> int:
    try:
        return max(1, len(os.sched_getaffinity(0)))
    except AttributeError:  # pragma: no cover
        return max(1, os.cpu_count() or 1)


def check_inputs(t, m, M, B) -> int:
    t, m, M, B, n, L, k = _batch(t, m, M, B)
    return lib().ppo_oracle_check_inputs(_f(t)[1], _f(m)[1], L, _f(M)[1], _f(B)[1], k, n)


def rank(order) -> int:
    o = np.ascontiguousarray(order, dtype=np.int32)
    return int(lib().ppo_oracle_rank(_i(o), len(o)))


def unrank(r: int, k: int) -> np.ndarray:
    o = np.zeros(k, dtype=np.int32)
    lib().ppo_oracle_unrank(int(r), k, _i(o))
    return o


def evaluate(t, m, M, B, order, cuts):
    """beta and feasibility of one explicit (ordering, cuts) solution of one instance."""
    t, m, M, B, n, L, k = _batch(t, m, M, B)
    assert n == 1
    o = np.ascontiguousarray(order, dtype=np.int32)
    c = np.ascontiguousarray(np.concatenate([np.asarray(cuts, dtype=np.int32), np.zeros(1, np.int32)]))
    beta = C.c_float()
    feas = C.c_int32()
    _check(lib().ppo_oracle_evaluate(_f(t)[1], _f(m)[1], L, _f(M)[1], _f(B)[1], k, _i(o), _i(c), C.byref(beta),
                                     C.byref(feas)))
    return np.float32(beta.value), bool(feas.value)


def _outputs(n, k):
    return (np.zeros(n, np.float32), np.zeros((n, max(k - 1, 0)), np.int32), np.zeros((n, k), np.int32))


def bruteforce(t, m, M, B):
    t, m, M, B, n, L, k = _batch(t, m, M, B)
    beta, cuts, order = _outputs(n, k)
    cbuf = np.zeros(max(k - 1, 1), np.int32)
    for j in range(n):
        b = C.c_float()
        o = np.zeros(k, np.int32)
        _check(lib().ppo_oracle_bruteforce(_f(t[j])[1], _f(m[j])[1], L, _f(M[j])[1], _f(B[j])[1], k, C.byref(b),
                                           _i(cbuf), _i(o)))
        beta[j] = b.value
        cuts[j] = cbuf[:k - 1]
        order[j] = o
    return beta, cuts, order


def exhaustive(t, m, M, B, n_threads=None, rank_range=None):
    """Returns beta [n], cuts [n,k-1], order [n,k], and the number of DP candidates examined."""
    t, m, M, B, n, L, k = _batch(t, m, M, B)
    beta, cuts, order = _outputs(n, k)
    cbuf = np.zeros((n, max(k - 1, 1)), np.int32)
    cand = C.c_uint64(0)
    nt = n_threads or default_threads()
    fp = lambda a: a.ctypes.data_as(C.POINTER(C.c_float))
    if rank_range is None:
        rc = lib().ppo_oracle_exhaustive(fp(t), fp(m), L, fp(M), fp(B), k, n, fp(beta), _i(cbuf), _i(order), nt,
                                         C.byref(cand))
    else:
        rc = lib().ppo_oracle_exhaustive_range(fp(t), fp(m), L, fp(M), fp(B), k, n, int(rank_range[0]),
                                               int(rank_range[1]), fp(beta), _i(cbuf), _i(order), nt, C.byref(cand))
    _check(rc)
    if k > 1:
        # the C side strides cuts by k-1
        cuts[:] = cbuf.reshape(-1)[: n * (k - 1)].reshape(n, k - 1)
    return beta, cuts, order, int(cand.value)


def eval_orderings(t, m, M, B, rank_begin, rank_end, n_threads=None):
    """beta of each ordering of ONE instance with rank in [rank_begin, rank_end)."""
    t, m, M, B, n, L, k = _batch(t, m, M, B)
    assert n == 1
    out = np.zeros(int(rank_end - rank_begin), np.float32)
    cand = C.c_uint64(0)
    fp = lambda a: a.ctypes.data_as(C.POINTER(C.c_float))
    _check(lib().ppo_oracle_eval_orderings(fp(t), fp(m), L, fp(M), fp(B), k, int(rank_begin), int(rank_end), fp(out),
                                           n_threads or default_threads(), C.byref(cand)))
    return out, int(cand.value)


def subset_dp(t, m, M, B, n_threads=None):
    t, m, M, B, n, L, k = _batch(t, m, M, B)
    beta, cuts, order = _outputs(n, k)
    cbuf = np.zeros((n, max(k - 1, 1)), np.int32)
    fp = lambda a: a.ctypes.data_as(C.POINTER(C.c_float))
    _check(lib().ppo_oracle_subset_dp(fp(t), fp(m), L, fp(M), fp(B), k, n, fp(beta), _i(cbuf), _i(order),
                                      n_threads or default_threads()))
    if k > 1:
        cuts[:] = cbuf.reshape(-1)[: n * (k - 1)].reshape(n, k - 1)
    return beta, cuts, order
