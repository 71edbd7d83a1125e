"""oco_create_static: the same simulation with the state and the kernels' scratch in the library's
own device array instead of a caller-provided workspace -- for callers that cannot allocate.
Checked against oco_create's results (bit-identical: same kernels, same memory layout) and the
fp64 CPU reference, on two calls in a row, the second smaller than the first (it shares the
array with the first and must not see its contents)."""
import numpy as np
import pytest

from paper_2603_12617_amd import binding as B
from paper_2603_12617_amd import workloads as WL

pytestmark = pytest.mark.gpu

REG_RTOL, ABS_TOL = 1e-4, 1e-5


def _run(wl, data, static, chunk, n_max):
    sim = B.Simulation(wl, data, n_max=n_max, static=static)
    sim.run_all(chunk)
    out = dict(regret=sim.regret(), L=sim.cum_losses())
    out["W"], out["p"], out["wbar"] = (t.cpu().numpy() for t in sim.state())
    sim.close()
    return out


def _against_oracle(wl, data, got):
    from oracle import oracle as O
    ref = O.run_workload(wl, data, norm_every=0)
    assert (np.abs(got["regret"] - ref["regret"]) / np.maximum(np.abs(ref["regret"]), 1.0)).max() <= REG_RTOL
    assert (np.abs(got["L"] - ref["L"]) / np.maximum(np.abs(ref["L"]), 1.0)).max() <= REG_RTOL
    for k in ("W", "p", "wbar"):
        assert np.abs(got[k] - ref[k]).max() <= ABS_TOL, k


CASES = [
    # first call, then a smaller one of the same kind (smaller state, shorter call)
    [("c3", dict(T=700, R=6, d=300, K=9, seg_len=100), 256), ("c3", dict(T=200, R=2, d=64, K=3, seg_len=50), 64)],
    [("c5", dict(T=900, R=3, d=4096, K=8, wstar_nnz=64), 512), ("c5", dict(T=300, R=2, d=1024, K=4, nnz=8, wstar_nnz=16), 128)],
    [("c4", dict(T=300, R=70, d=256, K=16), 0), ("c2", dict(T=150, R=3, d=40, K=5), 50)],      # windowed kernel, then per-run streams
    [("c3", dict(T=400, R=3, d=200, K=5, seg_len=64, optimistic=True), 128), ("c1", dict(T=100, d=10, R=1), 0)],
]


@pytest.mark.parametrize("pair", CASES)
def test_static_workspace_gives_the_results_of_a_caller_workspace(pair):
    for name, over, chunk in pair:                       # two calls in a row on the one shared array
        wl = WL.make(name, **over)
        data = WL.generate(wl)
        print("case static", name, over, flush=True)
        got = _run(wl, data, True, chunk, chunk)
        want = _run(wl, data, False, chunk, chunk)
        for k in ("regret", "L", "W", "p", "wbar"):
            assert np.array_equal(got[k], want[k]), (name, k)
        _against_oracle(wl, data, got)


def test_static_workspace_limits_and_refusals():
    wl = WL.make("c4", T=64, R=1024, d=4096, K=16)       # 268 MB of iterates
    cfg, keep = B.make_config(d=wl.d, K=wl.K, T=wl.T, R=wl.R, D=wl.D, G=wl.G, eta=wl.eta, eps=wl.eps, loss=wl.loss)
    with pytest.raises(B.OcoError) as e:
        B.oco_create_static(cfg)
    assert e.value.status == B.OCO_ENOMEM
    wl = WL.make("c2", T=100, R=2, d=16, K=3)
    data = WL.generate(wl)
    sim = B.Simulation(wl, data, static=True)
    with pytest.raises(B.OcoError) as e:
        B.oco_set_timing(sim.h, True)                    # would create events
    assert e.value.status == B.OCO_EUNSUPPORTED
    sim.run_all()
    first = sim.regret().copy()
    sim.reset()
    sim.run_all(30)
    assert np.array_equal(sim.regret(), first)
    sim.close()
