"""The seeded input generator: determinism, shapes, and the value distributions the
benchmark configurations state."""
import math

import numpy as np
import pytest

from paper_2603_12617_amd import workloads as WL


def test_named_workloads_have_the_benchmark_shapes():
    shapes = {n: (WL.make(n).R, WL.make(n).K, WL.make(n).d, WL.make(n).T) for n in WL.names()}
    assert shapes == {"c1": (1, 1, 10, 1000), "c2": (64, 15, 100, 10000),
                      "c3": (256, 17, 1000, 100000), "c4": (1024, 16, 4096, 20000),
                      "c5": (16, 8, 1 << 20, 100000)}
    c2 = WL.make("c2")
    assert abs(c2.eta[0] - 0.01) < 1e-15 and abs(c2.eta[14] - 163.84) < 1e-10
    assert WL.make("c1").eps == 0.0 and WL.make("c5").nnz == 32


def test_generation_is_deterministic_and_run_keyed():
    wl = WL.make("c2", T=50, R=3, d=8)
    a, b = WL.generate(wl), WL.generate(wl)
    for k in ("x", "y", "u"):
        assert np.array_equal(a[k], b[k])
    # run r of a larger batch equals run r of a smaller one
    c = WL.generate(WL.make("c2", T=50, R=2, d=8))
    assert np.array_equal(c["x"], a["x"][:2]) and np.array_equal(c["y"], a["y"][:2])
    d = WL.generate(WL.make("c2", T=50, R=3, d=8, seed=1))
    assert not np.array_equal(d["x"], a["x"])


def test_config1_stream():
    wl = WL.make("c1")
    dat = WL.generate(wl)
    g = dat["x"].astype(np.float64)
    assert g.shape == (1000, 10) and dat["y"] is None
    np.testing.assert_allclose(np.linalg.norm(g, axis=1), wl.G, rtol=2e-7)
    u = dat["u"][0, 0].astype(np.float64)
    assert abs(np.linalg.norm(u) - wl.D) < 2e-7
    S = g.sum(0)
    # best fixed point in hindsight: no point of the ball has smaller total loss
    assert abs(S @ u + wl.D * np.linalg.norm(S)) < 1e-5
    v = np.random.default_rng(0).standard_normal((100, 10))
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    assert (v @ S >= S @ u - 1e-9).all()


def test_dense_squared_streams():
    wl = WL.make("c2", T=4000, R=2, d=50)
    dat = WL.generate(wl)
    assert dat["x"].shape == (2, 4000, 50) and dat["x"].dtype == np.float32
    assert abs(dat["x"].var() * wl.d - 1) < 0.02
    np.testing.assert_allclose(np.linalg.norm(dat["u"][:, 0].astype(np.float64), axis=1), 0.5, rtol=1e-6)
    resid = dat["y"] - np.einsum("rd,rtd->rt", dat["u"][:, 0], dat["x"])
    assert abs(resid.std() - 0.1) < 0.01 and abs(resid.mean()) < 0.01


def test_piecewise_stationary_comparator():
    wl = WL.make("c3", T=1000, R=2, d=40, seg_len=250)
    dat = WL.generate(wl)
    assert dat["u"].shape == (2, 4, 40) and list(dat["seg_start"]) == [0, 250, 500, 750]
    np.testing.assert_allclose(np.linalg.norm(dat["u"].astype(np.float64), axis=2), 0.8, rtol=1e-6)
    assert dat["x"].shape == (1000, 40)                       # shared across runs
    for s in range(4):
        sl = slice(250 * s, 250 * (s + 1))
        resid = dat["y"][0, sl] - dat["x"][sl] @ dat["u"][0, s]
        assert resid.std() < 0.13                               # labels follow the segment's w*
    wrong = dat["y"][0, 250:500] - dat["x"][250:500] @ dat["u"][0, 0]
    assert wrong.std() > 0.13


def test_logistic_labels_and_flip_rate():
    wl = WL.make("c4", T=20000, R=2, d=32)
    dat = WL.generate(wl)
    assert set(np.unique(dat["y"])) == {-1.0, 1.0}
    clean = np.where(dat["x"] @ dat["u"][:, 0].T >= 0, 1.0, -1.0).T
    rate = (clean != dat["y"]).mean()
    assert abs(rate - 0.1) < 0.01
    np.testing.assert_allclose(np.linalg.norm(dat["u"][:, 0].astype(np.float64), axis=1), 1.0, rtol=1e-6)


def test_sparse_rows():
    wl = WL.make("c5", T=3000, R=2, d=4096, wstar_nnz=64)
    dat = WL.generate(wl)
    col, val = dat["col"], dat["val"]
    assert col.shape == (3000, 32) and col.dtype == np.int32 and dat["x"] is None
    assert (np.diff(col, axis=1) > 0).all()                    # distinct and ascending
    assert col.min() >= 0 and col.max() < wl.d
    assert abs(val.var() * 32 - 1) < 0.03
    assert ((dat["u"] != 0).sum(axis=2) == 64).all()
    np.testing.assert_allclose(np.linalg.norm(dat["u"].astype(np.float64), axis=2), 0.5, rtol=1e-6)
    clean = (dat["u"][0, 0][col].astype(np.float64) * val).sum(1)
    assert abs((dat["y"][0] - clean).std() - 0.1) < 0.01


def test_run_slice():
    wl = WL.make("c2", T=20, R=4, d=5)
    dat = WL.generate(wl)
    sub_wl, sub = WL.run_slice(wl, dat, [3, 1])
    assert sub_wl.R == 2 and np.array_equal(sub["x"][0], dat["x"][3]) and np.array_equal(sub["y"][1], dat["y"][1])
