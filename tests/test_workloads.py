"""The seeded input generators: shapes, determinism, and the structure each workload promises."""
import math

import numpy as np
import pytest

from paper_2210_12219_amd import workloads as W

SHAPES = {"tiny": (256, 12, 4), "resnet50_shaped": (1024, 50, 6), "transformer_encoder": (4096, 96, 8),
          "headline": (64, 100, 10), "large": (1, 64, 11)}
FACTOR = {"tiny": 1.5, "resnet50_shaped": 1.3, "transformer_encoder": 1.25, "headline": 1.2, "large": 1.1}


@pytest.mark.parametrize("name", list(SHAPES))
def test_shapes_and_structure(name):
    n_full, L, k = SHAPES[name]
    n = min(n_full, 64)
    w = W.WORKLOADS[name](n_inst=n)
    assert (w.n_inst, w.L, w.k) == (n, L, k)
    assert w.t.shape == (n, L) and w.m.shape == (n, L) and w.M.shape == (n, k) and w.B.shape == (n, k, k)
    for a in (w.t, w.m, w.M, w.B):
        assert a.dtype == np.float32 and a.flags.c_contiguous and np.isfinite(a).all()
    assert (w.t > 0).all() and (w.m > 0).all() and (w.M > 0).all()
    assert np.array_equal(w.B, np.transpose(w.B, (0, 2, 1)))
    off = ~np.eye(k, dtype=bool)
    assert (w.B[:, off] > 0).all() and (w.B[:, ~off] == 0).all()
    np.testing.assert_allclose(w.M.sum(1), FACTOR[name] * w.m.astype(np.float64).sum(1), rtol=1e-5)
    assert w.orderings_per_instance == math.factorial(k)
    again = W.WORKLOADS[name](n_inst=n)
    for a, b in zip((w.t, w.m, w.M, w.B), (again.t, again.m, again.M, again.B)):
        assert np.array_equal(a, b)


def test_value_ranges():
    h = W.headline()
    assert h.t.min() >= 0.5 and h.t.max() <= 40 and h.m.min() >= 0.1 and h.m.max() <= 100
    iu = np.triu_indices(10, 1)
    b = h.B[:, iu[0], iu[1]]
    assert b.min() >= 1 and b.max() <= 100
    ratios = h.M / h.M.min(axis=1, keepdims=True)
    assert np.isin(np.round(ratios, 3), [1, 2, 4, 8]).all()
    lg = W.large()
    assert lg.t[0, :8].min() >= 20 and lg.t[0, 8:].max() <= 10 and (np.diff(lg.m[0]) >= 0).all()
    tr = W.transformer_encoder(n_inst=2)
    assert set(np.unique(tr.t).tolist()) == {16.0, 64.0}
    rn = W.resnet50_shaped(n_inst=2)
    assert 25.69 * 0.8 <= rn.t[0, 1] <= 25.69 * 1.2 and abs(rn.m[0, -1] - 8.192) < 1e-3


def test_quantised_random_instances_have_ties():
    w = W.random_instances(3, 20, 8, 3, quantised=True)
    assert len(np.unique(w.t)) <= 4 and (w.M == np.floor(w.M)).all()
