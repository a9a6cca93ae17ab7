"""Seeded synthetic workloads for the partition-and-placement search.

This module only draws random inputs. It contains none of the method's
arithmetic (no prefix sums, no feasibility test, no latency quotient), so both
the HIP path and the CPU oracle may take their inputs from it.

Every workload is a batch of independent instances of the problem the paper
states in Sec. I and Sec. III-B: a chain of L layers with weight sizes m and
boundary transfer sizes t, and a cluster of k nodes with memory capacities M
and a symmetric bandwidth matrix B (the complete communication graph G_c of
Sec. III).  The paper evaluates on Keras model-zoo chains (Sec. IV); those
models are not available here, so the five workloads below are synthetic
stand-ins with chains of similar length and value ranges.

Arrays returned (all float32, C-contiguous):
    t [n_inst, L]     size of the tensor leaving layer i (Mbit); t[:, L-1] unused
    m [n_inst, L]     weight size of layer i (MB)
    M [n_inst, k]     node memory capacity (MB)
    B [n_inst, k, k]  bandwidth between nodes (Mbps), exactly symmetric, diagonal 0

Draw order per instance is t, m, M, B from one numpy Generator per workload;
values are produced in float64 and cast to float32 last.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    L: int
    k: int
    n_inst: int
    seed: int
    t: np.ndarray
    m: np.ndarray
    M: np.ndarray
    B: np.ndarray

    @property
    def orderings_per_instance(self) -> int:
        f = 1
        for i in range(2, self.k + 1):
            f *= i
        return f

    @property
    def total_orderings(self) -> int:
        return self.n_inst * self.orderings_per_instance

    def take(self, n: int) -> "Workload":
        """The first n instances as a workload of their own."""
        n = min(n, self.n_inst)
        return Workload(self.name, self.L, self.k, n, self.seed,
                        np.ascontiguousarray(self.t[:n]), np.ascontiguousarray(self.m[:n]),
                        np.ascontiguousarray(self.M[:n]), np.ascontiguousarray(self.B[:n]))


def _log_uniform(rng: np.random.Generator, lo: float, hi: float, size) -> np.ndarray:
    return np.exp(rng.uniform(np.log(lo), np.log(hi), size))


def _symmetric_bandwidth(rng: np.random.Generator, k: int, lo: float, hi: float) -> np.ndarray:
    """Upper triangle drawn log-uniformly, mirrored to the lower triangle."""
    B = np.zeros((k, k), dtype=np.float64)
    iu = np.triu_indices(k, 1)
    B[iu] = _log_uniform(rng, lo, hi, len(iu[0]))
    B = B + B.T
    return B


def _scaled_uniform_capacity(rng: np.random.Generator, k: int, m: np.ndarray, factor: float) -> np.ndarray:
    """Capacities uniform in [0.5, 1.5], rescaled so that they sum to factor * sum(m)."""
    raw = rng.uniform(0.5, 1.5, k)
    return raw * (factor * float(np.sum(m)) / float(np.sum(raw)))


def _finish(name, L, k, n_inst, seed, ts, ms, Ms, Bs) -> Workload:
    t = np.ascontiguousarray(np.stack(ts).astype(np.float32))
    m = np.ascontiguousarray(np.stack(ms).astype(np.float32))
    M = np.ascontiguousarray(np.stack(Ms).astype(np.float32))
    B64 = np.stack(Bs)
    B = np.ascontiguousarray(B64.astype(np.float32))
    # the cast is element-wise, so symmetry of the float64 matrix carries over bit for bit
    assert np.array_equal(B, np.transpose(B, (0, 2, 1)))
    return Workload(name, L, k, n_inst, seed, t, m, M, B)


def tiny(n_inst: int = 256, seed: int = 0) -> Workload:
    """256 x (L=12, k=4); small enough for brute force over every (cut set, permutation)."""
    L, k = 12, 4
    rng = np.random.default_rng(seed)
    ts, ms, Ms, Bs = [], [], [], []
    for _ in range(n_inst):
        t = _log_uniform(rng, 0.1, 20.0, L)
        m = _log_uniform(rng, 0.05, 50.0, L)
        ts.append(t); ms.append(m)
        Ms.append(_scaled_uniform_capacity(rng, k, m, 1.5))
        Bs.append(_symmetric_bandwidth(rng, k, 2.0, 50.0))
    return _finish("tiny", L, k, n_inst, seed, ts, ms, Ms, Bs)


def _resnet50_chain():
    """Stage-wise activation sizes (Mbit, fp32) and weight sizes (MB, fp32) of a 50-layer
    bottleneck-block chain: stem, then 9/12/18/9 convolutions in four stages, then the head."""
    mbit = lambda h, w, c: h * w * c * 32 / 1e6
    t = [mbit(56, 56, 64)]
    mw = [7 * 7 * 3 * 64 * 4 / 1e6]
    stages = [(9, 64, mbit(56, 56, 256)), (12, 128, mbit(28, 28, 512)),
              (18, 256, mbit(14, 14, 1024)), (9, 512, mbit(7, 7, 2048))]
    for n_layers, c, act in stages:
        for j in range(n_layers):
            t.append(act)
            params = (4 * c * c, 9 * c * c, 4 * c * c)[j % 3]
            mw.append(params * 4 / 1e6)
    t.append(1000 * 32 / 1e6)
    mw.append(2048 * 1000 * 4 / 1e6)
    return np.array(t), np.array(mw)


def resnet50_shaped(n_inst: int = 1024, seed: int = 1) -> Workload:
    """1024 x (L=50, k=6); activation sizes jittered by +-20 % per instance."""
    L, k = 50, 6
    base_t, base_m = _resnet50_chain()
    assert len(base_t) == L and len(base_m) == L
    rng = np.random.default_rng(seed)
    ts, ms, Ms, Bs = [], [], [], []
    for _ in range(n_inst):
        t = base_t * rng.uniform(0.8, 1.2, L)
        m = base_m.copy()
        ts.append(t); ms.append(m)
        Ms.append(_scaled_uniform_capacity(rng, k, m, 1.3))
        Bs.append(_symmetric_bandwidth(rng, k, 2.0, 50.0))
    return _finish("resnet50_shaped", L, k, n_inst, seed, ts, ms, Ms, Bs)


def transformer_encoder(n_inst: int = 4096, seed: int = 2) -> Workload:
    """4096 x (L=96, k=8); 24 blocks of (attention, add&norm, FFN-up, FFN-down).
    No jitter on t, so almost every ordering ties on the bottleneck latency."""
    L, k = 96, 8
    base_t = np.tile(np.array([16.0, 16.0, 64.0, 16.0]), 24)
    base_m = np.tile(np.array([16.0, 2.0 ** -7, 16.0, 16.0]), 24)
    rng = np.random.default_rng(seed)
    ts, ms, Ms, Bs = [], [], [], []
    for _ in range(n_inst):
        ts.append(base_t.copy()); ms.append(base_m.copy())
        Ms.append(_scaled_uniform_capacity(rng, k, base_m, 1.25))
        Bs.append(_symmetric_bandwidth(rng, k, 2.0, 50.0))
    return _finish("transformer_encoder", L, k, n_inst, seed, ts, ms, Ms, Bs)


def headline(n_inst: int = 64, seed: int = 3) -> Workload:
    """64 x (L=100, k=10): 3,628,800 orderings per instance; the benchmarked workload."""
    L, k = 100, 10
    rng = np.random.default_rng(seed)
    ts, ms, Ms, Bs = [], [], [], []
    for _ in range(n_inst):
        t = _log_uniform(rng, 0.5, 40.0, L)
        m = _log_uniform(rng, 0.1, 100.0, L)
        raw = rng.choice(np.array([1.0, 2.0, 4.0, 8.0]), size=k)
        ts.append(t); ms.append(m)
        Ms.append(raw * (1.2 * float(np.sum(m)) / float(np.sum(raw))))
        Bs.append(_symmetric_bandwidth(rng, k, 1.0, 100.0))
    return _finish("headline", L, k, n_inst, seed, ts, ms, Ms, Bs)


def large(n_inst: int = 1, seed: int = 4) -> Workload:
    """1 x (L=64, k=11): 39,916,800 orderings, tight capacities, most orderings infeasible."""
    L, k = 64, 11
    rng = np.random.default_rng(seed)
    ts, ms, Ms, Bs = [], [], [], []
    for _ in range(n_inst):
        t = np.concatenate([_log_uniform(rng, 20.0, 100.0, 8), _log_uniform(rng, 0.5, 10.0, L - 8)])
        m = np.sort(_log_uniform(rng, 1.0, 400.0, L))
        ts.append(t); ms.append(m)
        Ms.append(_scaled_uniform_capacity(rng, k, m, 1.1))
        Bs.append(_symmetric_bandwidth(rng, k, 1.0, 100.0))
    return _finish("large", L, k, n_inst, seed, ts, ms, Ms, Bs)


WORKLOADS = {
    "tiny": tiny,
    "resnet50_shaped": resnet50_shaped,
    "transformer_encoder": transformer_encoder,
    "headline": headline,
    "large": large,
}


def random_instances(seed: int, n_inst: int, L: int, k: int, *, capacity_factor: float = 1.5,
                     quantised: bool = False) -> Workload:
    """Small random batches for tests.  With quantised=True, t, m and B take few distinct small
    integer values (so equal latencies and exact capacity hits occur) and capacities are integers."""
    rng = np.random.default_rng(seed)
    ts, ms, Ms, Bs = [], [], [], []
    for _ in range(n_inst):
        if quantised:
            t = rng.integers(1, 5, L).astype(np.float64)
            m = rng.integers(1, 6, L).astype(np.float64)
            cap = np.floor(rng.uniform(0.5, 1.5, k) * capacity_factor * m.sum() / k)
            B = np.zeros((k, k))
            iu = np.triu_indices(k, 1)
            B[iu] = rng.integers(1, 4, len(iu[0])).astype(np.float64)
            B = B + B.T
        else:
            t = _log_uniform(rng, 0.1, 20.0, L)
            m = _log_uniform(rng, 0.05, 50.0, L)
            cap = _scaled_uniform_capacity(rng, k, m, capacity_factor)
            B = _symmetric_bandwidth(rng, k, 2.0, 50.0)
        ts.append(t); ms.append(m); Ms.append(cap); Bs.append(B)
    return _finish("random", L, k, n_inst, seed, ts, ms, Ms, Bs)


# ---------------------------------------------------------------------------------------------
# Cluster form: more nodes than segments.  Same arrays, with k read as the cluster size n.
# ---------------------------------------------------------------------------------------------
_SHANNON_A = 283230.0   # Sec. IV: chosen so that a device 80 m from the router gets 5.5 Mbps


def _geometric_bandwidth(rng: np.random.Generator, n: int) -> np.ndarray:
    """Sec. IV, Eq. 12: device positions with |x|, |y| uniform in (1, 150) m and a random sign each,
    rate of a device r = log2(1 + a / (x^2 + y^2)).  The paper gives the rate as a function of ONE
    position (relative to the router) but needs a weight per PAIR of devices; the reading taken here
    is that traffic between two devices passes the router, so the pair gets the lower of the two
    rates."""
    mag = rng.uniform(1.0, 150.0, (n, 2))
    sign = rng.choice(np.array([-1.0, 1.0]), size=(n, 2))
    pos = mag * sign
    r = np.log2(1.0 + _SHANNON_A / np.sum(pos * pos, axis=1))
    B = np.minimum(r[:, None], r[None, :])
    np.fill_diagonal(B, 0.0)
    return B


def cluster_geometric(n: int, capacity_mb: float, n_inst: int = 16, seed: int = 5) -> Workload:
    """The paper's evaluation cluster (Sec. IV): n randomly placed devices of ONE capacity (64, 128, 256
    or 512 MB there) under the 50-layer bottleneck-block chain of resnet50_shaped (about 94 MB of
    weights), activation sizes jittered by +-20 % per instance.  Bandwidths come in few distinct
    values (each device's rate), so equal latencies are common."""
    L = 50
    base_t, base_m = _resnet50_chain()
    rng = np.random.default_rng(seed)
    ts, ms, Ms, Bs = [], [], [], []
    for _ in range(n_inst):
        ts.append(base_t * rng.uniform(0.8, 1.2, L)); ms.append(base_m.copy())
        Ms.append(np.full(n, float(capacity_mb)))
        Bs.append(_geometric_bandwidth(rng, n))
    return _finish(f"cluster_geometric_n{n}_c{int(capacity_mb)}", L, n, n_inst, seed, ts, ms, Ms, Bs)


def cluster_mixed(n: int, L: int = 100, n_inst: int = 8, seed: int = 6, capacity_factor: float = 0.25) -> Workload:
    """n nodes with capacities of 1x, 2x, 4x or 8x a unit (each about capacity_factor of the model on
    average) and log-uniform bandwidths, under a log-uniform chain as in `headline`: at least
    1/capacity_factor segments are needed, and which nodes to leave out is part of the search."""
    rng = np.random.default_rng(seed)
    ts, ms, Ms, Bs = [], [], [], []
    for _ in range(n_inst):
        t = _log_uniform(rng, 0.5, 40.0, L)
        m = _log_uniform(rng, 0.1, 100.0, L)
        raw = rng.choice(np.array([1.0, 2.0, 4.0, 8.0]), size=n)
        ts.append(t); ms.append(m)
        Ms.append(raw * (capacity_factor * float(np.sum(m)) / float(np.mean(raw))))
        Bs.append(_symmetric_bandwidth(rng, n, 1.0, 100.0))
    return _finish(f"cluster_mixed_n{n}", L, n, n_inst, seed, ts, ms, Ms, Bs)


# ---------------------------------------------------------------------------------------------
# Compute stages (Sec. I, Eq. 1): per-layer work and per-node speed beside a workload's arrays.
# ---------------------------------------------------------------------------------------------
def compute_terms(w: Workload, seed: int = 7, seconds: float = 1.0, quantised: bool = False):
    """(work [n_inst, L], speed [n_inst, k]) float32 for the instances of w.  The paper gives one data
    point (ResNet50 on a Raspberry Pi 4: 225 ms for the whole model, 7.5 times less than one average
    transfer) and no per-layer figures, so these are synthetic: work per layer log-uniform over a
    factor of 30, speeds 1x, 2x or 4x a unit, scaled so that the whole model takes `seconds` on a node
    of speed 1.  With quantised=True both take few small integer values (equal stage times occur)."""
    rng = np.random.default_rng(seed)
    if quantised:
        work = rng.integers(1, 5, (w.n_inst, w.L)).astype(np.float64)
        speed = rng.integers(1, 4, (w.n_inst, w.k)).astype(np.float64)
    else:
        work = np.exp(rng.uniform(np.log(1.0), np.log(30.0), (w.n_inst, w.L)))
        work *= seconds / work.sum(axis=1, keepdims=True)
        speed = rng.choice(np.array([1.0, 2.0, 4.0]), size=(w.n_inst, w.k))
    return np.ascontiguousarray(work, dtype=np.float32), np.ascontiguousarray(speed, dtype=np.float32)
