#!/usr/bin/env python3
"""Host-side check of the jump tables of the paired enumeration kernel (run by build.py and by the CPU tests).

ppo_pair_program.h turns the memory windows of a (node, DP row) into the 16-bit offsets that the generated code's
headers jump to.  A wrong table could send a wave anywhere, so the very function the kernel uses is compiled for
the host here and every table it makes is walked through a model of the generated code (what sits at which
offset: ppo_pair_layout.json, itself verified against the compiled kernel by check_pair_code.py):
  - every jump lands on the start of a chain, a +inf, a piece of run code or the end of the block;
  - the walk ends, within as many jumps as a row has outputs;
  - the registers then hold, for every output, the minimum over its window of the values they held before
    (random 16-bit values), and only the outputs wanted were written.
"""
import ctypes
import json
import os
import subprocess
import sys
import tempfile

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SHIM = r'''
#include "ppo_pair_program.h"
extern "C" void pair_row_program_host(int L, int k, int s, const unsigned char* lo_row, uint16_t* entry) {
    ppo::pair_row_program(L, k, s, lo_row, entry);
}
'''


def load_builder(tmpdir):
    src, lib = os.path.join(tmpdir, "shim.cpp"), os.path.join(tmpdir, "shim.so")
    open(src, "w").write(SHIM)
    subprocess.check_call([os.environ.get("CXX", "g++"), "-O1", "-std=c++17", "-shared", "-fPIC", "-I", HERE, "-o", lib, src])
    dll = ctypes.CDLL(lib)
    dll.pair_row_program_host.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 2
    dll.pair_row_program_host.restype = None
    return dll


class Model:
    """what the generated code does from a given offset on, up to the header that follows"""

    def __init__(self):
        lay = json.load(open(os.path.join(HERE, "ppo_pair_layout.json")))
        self.nslot, self.umax, self.end = lay["nslot"], lay["umax"], lay["end"] // 4
        self.at = {}
        for us, by_w in lay["entries"].items():
            for ws, off in by_w.items():
                assert off % 4 == 0 and off // 4 not in self.at
                self.at[off // 4] = ("chain", int(us), int(ws))
        for ps, by_a in lay["runs"].items():
            for as_, off in by_a.items():
                assert off % 4 == 0 and off // 4 not in self.at
                self.at[off // 4] = ("run", int(as_), int(ps))

    def walk(self, entry, top, regs):
        """follows the table from the row's highest output; returns the number of jumps"""
        pos, jumps = top, 0
        while True:
            target = int(entry[(pos - 1) % self.nslot])
            jumps += 1
            assert jumps <= top + 2, "the walk does not end"
            if target == self.end:
                return jumps
            assert target in self.at, f"jump to +{4 * target}: nothing starts there"
            kind, a, b = self.at[target]
            if kind == "chain":
                u, w = a, b
                regs[u] = min(regs[u - w + 1:u + 1]) if w else 0x7C00
                pos = u - 1
            else:
                for x in range(a, b + 1):
                    regs[x] = min(regs[x - 1], regs[x])
                pos = b - 1


def check_row(dll, model, rng, L, k, s, lo_row):
    entry = np.zeros(model.nslot, dtype=np.uint16)
    lo = np.ascontiguousarray(lo_row, dtype=np.uint8)
    dll.pair_row_program_host(L, k, s, lo.ctypes.data, entry.ctypes.data)
    top = L - k + 1
    before = [0] + [int(x) for x in rng.integers(0x0400, 0x7C00, size=model.umax)]
    regs = list(before)
    jumps = model.walk(entry, top, regs)
    wanted = [top] if s == k - 1 else range(1, top + 1)
    for u in range(1, model.umax + 1):
        if u in wanted:
            e = u + s
            first = max(int(lo[e]), s)
            w = max(e - first, 0)
            want = min(before[u - w + 1:u + 1]) if w else 0x7C00
        else:
            want = before[u]
        assert regs[u] == want, f"L={L} k={k} s={s} output {u}: {regs[u]:#x}, expected {want:#x}"
    return jumps


def random_windows(rng, L, kind):
    """lo[0..L] of one node: non-decreasing, lo[e] <= e (lo[e] = e: not even layer e-1 fits)"""
    if kind == 0:     # a memory limit over random weights
        m = np.exp(rng.uniform(np.log(0.1), np.log(100.0), size=L))
        cap = rng.uniform(0.02, 0.6) * m.sum()
        P = np.concatenate([[0.0], np.cumsum(m)])
        lo = np.zeros(L + 1, dtype=np.int64)
        for e in range(L + 1):
            i = 0
            while P[e] - P[i] > cap:
                i += 1
            lo[e] = i
        return lo
    if kind == 1:     # everything fits
        return np.zeros(L + 1, dtype=np.int64)
    if kind == 2:     # a sliding window of fixed width
        width = int(rng.integers(1, 12))
        return np.maximum(np.arange(L + 1) - width, 0)
    if kind == 3:     # nothing fits at some ends
        lo = np.maximum(np.arange(L + 1) - int(rng.integers(1, 6)), 0)
        for e in rng.integers(1, L + 1, size=4):
            lo[e:] = np.maximum(lo[e:], e)
        return np.minimum(lo, np.arange(L + 1))
    steps = rng.integers(0, 3, size=L + 1) * (rng.random(L + 1) < 0.4)   # irregular steps
    return np.minimum(np.cumsum(steps), np.arange(L + 1))


def run_checks(n_random=400, seed=0):
    rng = np.random.default_rng(seed)
    model = Model()
    rows = jumps = 0
    with tempfile.TemporaryDirectory() as d:
        dll = load_builder(d)
        shapes = [(100, 10), (96, 8), (64, 11), (50, 6), (100, 6), (12, 6), (6, 6), (7, 6), (106, 12), (101, 7)]
        for n in range(n_random):
            L, k = shapes[n % len(shapes)] if n < 4 * len(shapes) else (0, 0)
            if L == 0:
                k = int(rng.integers(6, 13))
                L = int(rng.integers(k, min(128, k + 94) + 1))
            lo = random_windows(rng, L, n % 5)
            for s in range(1, k):
                jumps += check_row(dll, model, rng, L, k, s, lo)
                rows += 1
    return rows, jumps


if __name__ == "__main__":
    r, j = run_checks(int(sys.argv[1]) if len(sys.argv) > 1 else 400)
    print(f"paired kernel: {r} jump tables walked through the model of the generated code, {j} jumps, all end and give the window minima")
