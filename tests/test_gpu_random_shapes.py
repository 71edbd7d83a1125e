"""Seeded random shapes against the oracle: dimensions that are not round numbers, every loss,
shared and per-run streams, plain and optimistic updates, moving comparators, and a random way of
cutting the horizon into calls (dense results must not depend on it at all; sparse ones only to
rounding unless every cut is a multiple of 64)."""
import numpy as np
import pytest

from paper_2603_12617_amd import binding as B
from paper_2603_12617_amd import workloads as WL

pytestmark = pytest.mark.gpu

REG_RTOL = 1e-4     # regret, relative to max(|regret|, 1)
ABS_TOL = 1e-5      # iterates, combined iterate, Hedge weights


def _run(wl, data, cuts):
    sim = B.Simulation(wl, data)
    t = 0
    for c in cuts:
        sim.run(t, c)
        t += c
    assert t == wl.T
    out = dict(regret=sim.regret(), L=sim.cum_losses())
    out["W"], out["p"], out["wbar"] = (x.cpu().numpy() for x in sim.state())
    sim.close()
    return out


def _cuts(rng, T, multiple=1):
    cuts, t = [], 0
    while t < T:
        c = int(rng.integers(1, max(2, T // 3)))
        c = max(multiple, c // multiple * multiple)
        c = min(c, T - t)
        cuts.append(c)
        t += c
    return cuts


def _compare(wl, data, got, label):
    from oracle import oracle as O
    ref = O.run_workload(wl, data, norm_every=0 if wl.nnz else None)
    dreg = np.abs(got["regret"] - ref["regret"]) / np.maximum(np.abs(ref["regret"]), 1.0)
    dL = np.abs(got["L"] - ref["L"]) / np.maximum(np.abs(ref["L"]), 1.0)
    print("%s regret rel %.2e L rel %.2e W %.2e p %.2e wbar %.2e" % (
        label, dreg.max(), dL.max(), np.abs(got["W"] - ref["W"]).max(), np.abs(got["p"] - ref["p"]).max(),
        np.abs(got["wbar"] - ref["wbar"]).max()), flush=True)
    assert dreg.max() <= REG_RTOL and dL.max() <= REG_RTOL, label
    for k in ("W", "p", "wbar"):
        assert np.abs(got[k] - ref[k]).max() <= ABS_TOL, (label, k)


@pytest.mark.parametrize("case", range(48))
def test_random_dense_shapes(case):
    rng = np.random.default_rng(1000 + case)
    d = int(rng.choice([1, 2, 3, 7, 63, 64, 65, 100, 129, 257, 511, 640, 1000, 1025, 2047, 2050, 3001, 4093, 4096]))
    K = int(rng.integers(1, 21))
    R = int(rng.integers(1, 7))
    T = int(rng.integers(65, 420))
    name = ["c1", "c2", "c3", "c4"][int(rng.integers(0, 4))]
    over = dict(d=d, K=K, R=R, T=T, x_shared=bool(rng.integers(0, 2)), optimistic=bool(rng.integers(0, 2)),
                seg_len=int(rng.choice([0, 1, 17, 64, 100])), seed=case)
    if name == "c1":
        over["seg_len"] = 0          # the linear workload's comparator is the best fixed point in hindsight
    wl = WL.make(name, **over)
    data = WL.generate(wl)
    print("case", case, name, over, flush=True)
    whole = _run(wl, data, [wl.T])
    _compare(wl, data, whole, "dense %d" % case)
    cuts = _cuts(rng, wl.T)
    part = _run(wl, data, cuts)
    for k in ("regret", "L", "W", "p", "wbar"):
        assert np.array_equal(whole[k], part[k]), (case, k, cuts)


@pytest.mark.parametrize("case", range(24))
def test_random_sparse_shapes(case):
    rng = np.random.default_rng(2000 + case)
    nnz = int(rng.choice([1, 3, 8, 17, 32, 64]))
    d = int(rng.choice([nnz + 1, 100, 777, 4096, 50000, 1 << 17]))
    d = max(d, nnz + 1)
    K = int(rng.integers(1, 13))
    R = int(rng.integers(1, 9))
    T = int(rng.integers(65, 500))
    over = dict(d=d, K=K, R=R, T=T, nnz=nnz, wstar_nnz=min(d, 64), seg_len=int(rng.choice([0, 50, 128])), seed=case)
    if case % 3 == 0:       # steps far larger than the ball: folds inside the launch segment
        over["eta"] = tuple(float(10.0 ** rng.uniform(-1, 3)) for _ in range(K))
    wl = WL.make("c5", **over)
    data = WL.generate(wl)
    print("case", case, over, flush=True)
    whole = _run(wl, data, [wl.T])
    _compare(wl, data, whole, "sparse %d" % case)
    # the same calls give the same bits; other cuts of the horizon (also at window boundaries: the
    # first window of a call is gathered after all earlier steps, later ones before the previous
    # window's) regroup float sums and agree to rounding
    cuts = _cuts(rng, wl.T, multiple=64)
    part = _run(wl, data, cuts)
    again = _run(wl, data, cuts)
    for k in ("regret", "L", "W", "p", "wbar"):
        assert np.array_equal(again[k], part[k]), (case, k)
    ragged = _run(wl, data, _cuts(rng, wl.T))
    for other in (part, ragged):
        for k in ("regret", "L", "W", "p", "wbar"):
            scale = max(1.0, float(np.abs(whole[k]).max()))
            np.testing.assert_allclose(other[k], whole[k], rtol=0, atol=2e-6 * scale, err_msg=k)
