"""The windowed dense path (windows of 64 rounds as contractions on the matrix cores, iterates in
registers or streamed from HBM) against the fp64 CPU reference, through the C ABI.  Same
tolerances as the other parity tests: regret 1e-4 relative, iterates / weights 1e-5 absolute."""
import numpy as np
import pytest

from paper_2603_12617_amd import binding as B
from paper_2603_12617_amd import workloads as WL
from test_gpu_parity import _check, _gpu

pytestmark = pytest.mark.gpu

WIN = dict(dense_path=2)

# ragged first / last windows, learners that do not fill the last tile of 16, one and many blocks
# of 16 coordinates per wavefront, d not a multiple of 16, K = 17, all three losses, comparator
# segments that cut windows
CASES = [
    ("c1", dict(T=130, d=4, R=2)),
    ("c1", dict(T=257, d=64, R=3)),
    ("c3", dict(T=500, R=3, d=100, K=15, seg_len=100)),
    ("c3", dict(T=333, R=2, d=28, K=4, seg_len=50)),
    ("c3", dict(T=65, R=2, d=4, K=2, seg_len=10)),
    ("c3", dict(T=1000, R=3, d=132, K=17, seg_len=100)),
    ("c3", dict(T=777, R=5, d=1000, K=17, seg_len=100)),
    ("c3", dict(T=300, R=2, d=260, K=3, seg_len=7)),
    ("c3", dict(T=300, R=2, d=2048, K=9, seg_len=64)),
    ("c4", dict(T=500, R=5, d=512, K=16)),
    ("c4", dict(T=301, R=3, d=4096, K=16)),
    ("c4", dict(T=150, R=2, d=3000, K=2)),
    ("c3", dict(T=100, R=1, d=48, K=64, seg_len=0)),
    ("c4", dict(T=200, R=40, d=1024, K=16)),                       # 40 tiles
]


@pytest.mark.parametrize("name,over", CASES)
@pytest.mark.parametrize("resident", [1, 0, 2, 3, 4])
def test_windowed_rounds_match_the_oracle(name, over, resident):
    wl = WL.make(name, **over)
    data = WL.generate(wl)
    print("case windowed", name, over, "resident", resident, flush=True)
    got = _gpu(wl, data, options=dict(WIN, window_resident=resident))
    _check(wl, data, got, label="windowed %s %s resident=%d" % (name, over, resident))


# the optimistic two-step update (Eq. (3)) in the windowed kernels that have it (two tiles per
# workgroup, streamed or in registers; loading wavefronts), base level only and both levels
@pytest.mark.parametrize("name,over", [
    ("c1", dict(T=257, d=64, R=3)),
    ("c3", dict(T=500, R=3, d=100, K=15, seg_len=100)),
    ("c3", dict(T=1000, R=3, d=132, K=17, seg_len=100)),
    ("c3", dict(T=300, R=2, d=2048, K=9, seg_len=64)),
    ("c4", dict(T=301, R=3, d=4096, K=16)),
    ("c4", dict(T=150, R=2, d=3000, K=2, eta=(0.5, 20.0))),
    ("c4", dict(T=130, R=3, d=8192, K=6)),
])
@pytest.mark.parametrize("resident", [0, 3, 4])
@pytest.mark.parametrize("optimistic", [1, 2])
def test_windowed_optimistic_rounds_match_the_oracle(name, over, resident, optimistic):
    wl = WL.make(name, optimistic=optimistic, **over)
    data = WL.generate(wl)
    print("case windowed optimistic", optimistic, name, over, "resident", resident, flush=True)
    got = _gpu(wl, data, options=dict(WIN, window_resident=resident))
    _check(wl, data, got, label="windowed optimistic %s %s resident=%d" % (name, over, resident))


@pytest.mark.parametrize("resident", [0, 3, 4])
def test_windowed_optimistic_results_and_how_the_horizon_is_cut(resident):
    """The hint of a call's first round needs the last row of the call before and the learners'
    hint scalars: both are kept in the state.  Different cuts regroup float32 sums (as without
    the optimistic update); the same cuts give the same bits."""
    wl = WL.make("c3", optimistic=1, T=400, R=2, d=1000, K=17, seg_len=90)
    data = WL.generate(wl)
    opt = dict(WIN, window_resident=resident)
    whole = _gpu(wl, data, options=opt)
    _check(wl, data, whole, label="windowed optimistic whole")
    for c in (64, 100, 37):
        part = _gpu(wl, data, chunk=c, n_max=c, options=opt)
        again = _gpu(wl, data, chunk=c, n_max=c, options=opt)
        _check(wl, data, part, label="windowed optimistic chunk %d" % c)
        for k in ("regret", "L", "W", "p", "wbar"):
            assert np.array_equal(part[k], again[k]), (k, c)
        scale = max(1.0, float(np.abs(whole["regret"]).max()))
        assert np.abs(part["regret"] - whole["regret"]).max() <= 2e-6 * scale * 10
        assert np.abs(part["W"] - whole["W"]).max() <= 2e-5


@pytest.mark.parametrize("name,over", [
    ("c3", dict(T=200, R=2, d=8192, K=5, seg_len=64)),
    ("c4", dict(T=130, R=3, d=16384, K=6)),
    ("c3", dict(T=70, R=1, d=65536, K=2, seg_len=0)),
])
def test_dimensions_beyond_one_wavefronts_registers(name, over):
    """d > 4096: the iterates cannot stay on chip; the same sweep streams them from HBM once per
    window.  This is the default (and only) dense path at these sizes."""
    wl = WL.make(name, **over)
    data = WL.generate(wl)
    print("case wide", name, over, flush=True)
    _check(wl, data, _gpu(wl, data), label="wide %s %s" % (name, over))


def test_steps_far_larger_than_the_ball_and_a_tiny_radius():
    """Every round lands far outside the ball: the projection factors of a window multiply to
    far below float32's range, which the window's scalars (float64) and its fold factor carry."""
    wl = WL.make("c3", T=200, R=2, d=20, K=3, eta=(1e4, 1e6, 3.0), D=1e-3, seg_len=0)
    data = WL.generate(wl)
    _check(wl, data, _gpu(wl, data, options=WIN), label="windowed huge eta")
    wl = WL.make("c4", T=200, R=2, d=64, K=4, eta=(1e-3, 1.0, 1e3, 1e8))
    data = WL.generate(wl)
    _check(wl, data, _gpu(wl, data, options=WIN), label="windowed logistic huge eta")


@pytest.mark.parametrize("name,over", [
    ("c3", dict(T=400, R=2, d=1000, K=17, seg_len=90)),
    ("c4", dict(T=300, R=2, d=4096, K=4)),
])
@pytest.mark.parametrize("resident", [1, 0, 2, 3, 4])
def test_windowed_results_and_how_the_horizon_is_cut(name, over, resident):
    """Repeated runs are bit-identical (every sum has a fixed order).  Different cuts of the horizon
    agree to float32 rounding: the first window of a call takes its inner products with the stored
    iterates, later ones through the window before (and a cut inside a window regroups sums)."""
    opt = dict(WIN, window_resident=resident)
    wl = WL.make(name, **over)
    data = WL.generate(wl)
    whole = _gpu(wl, data, options=opt)
    again = _gpu(wl, data, options=opt)
    for k in ("regret", "L", "W", "p", "wbar"):
        assert np.array_equal(whole[k], again[k]), k
    for c in (64, 128, 37, 1):
        print("case windowed", name, over, "chunk", c, flush=True)
        part = _gpu(wl, data, chunk=c, n_max=c, options=opt)
        for k in ("regret", "L", "W", "p", "wbar"):
            scale = max(1.0, float(np.abs(whole[k]).max()))
            np.testing.assert_allclose(part[k], whole[k], rtol=0, atol=2e-6 * scale, err_msg="%s %d" % (k, c))
    _check(wl, data, part, label="windowed %s chunk 1" % name)


def test_a_state_may_change_kernels_between_calls():
    """The register kernel leaves a lazily scaled iterate (sigma, V), the windowed one the iterate
    itself: either continues from the other's state."""
    wl = WL.make("c3", T=600, R=3, d=256, K=6, seg_len=100, eta=(0.01, 0.1, 1.0, 10.0, 100.0, 1000.0))
    data = WL.generate(wl)
    sim = B.Simulation(wl, data)
    for t0, n, path in ((0, 150, 1), (150, 170, 2), (320, 130, 1), (450, 150, 2)):
        B.oco_set_option(sim.h, "dense_path", path)
        sim.run(t0, n)
    got = dict(regret=sim.regret(), L=sim.cum_losses())
    got["W"], got["p"], got["wbar"] = (t.cpu().numpy() for t in sim.state())
    sim.close()
    _check(wl, data, got, label="mixed kernels")


def test_windowed_path_is_the_default_for_many_learners_on_a_shared_stream(capfd):
    wl = WL.make("c4", T=130, R=130, d=2048, K=16)            # 2080 learners
    data = WL.generate(wl)
    got = _gpu(wl, data, options=dict(verbose=1))
    assert "windowed contraction kernel" in capfd.readouterr().err
    _check(wl, data, got, runs=[0, 65, 129], label="windowed by default")


def test_option_errors():
    wl = WL.make("c2", T=100, R=2, d=16, K=3)                   # one stream per run
    data = WL.generate(wl)
    sim = B.Simulation(wl, data)
    with pytest.raises(B.OcoError) as e:
        B.oco_set_option(sim.h, "dense_path", 2)               # needs a shared stream
    assert e.value.status == B.OCO_EUNSUPPORTED
    for key, val in (("dense_path", 3), ("sparse_lpw", 5), ("meta_beside", 2), (99, 0), ("dense_wpb", 0), ("verbose", -2)):
        with pytest.raises(B.OcoError) as e:
            B.oco_set_option(sim.h, key, val)
        assert e.value.status == B.OCO_EINVAL, (key, val)
    B.oco_set_option(sim.h, "dense_wpb", 4)
    B.oco_set_option(sim.h, "dense_wpb", -1)                   # back to the library's choice
    sim.run_all()
    _check(wl, data, dict(regret=sim.regret(), L=sim.cum_losses(),
                          **dict(zip(("W", "p", "wbar"), (t.cpu().numpy() for t in sim.state())))), label="options")
    sim.close()
    wl = WL.make("c3", T=64, R=1, d=8192, K=2, seg_len=0)
    data = WL.generate(wl)
    sim = B.Simulation(wl, data)
    with pytest.raises(B.OcoError) as e:
        B.oco_set_option(sim.h, "dense_path", 1)               # does not fit one wavefront's registers
    assert e.value.status == B.OCO_EUNSUPPORTED
    with pytest.raises(B.OcoError) as e:
        B.oco_run_rounds(sim.h, 0, 10, x_ptr=sim.x.data_ptr() + 4, y=sim.y)   # rows not 16-byte aligned
    assert e.value.status == B.OCO_EUNSUPPORTED
    sim.close()
