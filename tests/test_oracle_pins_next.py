"""Pins for the parts of the CPU reference beyond the plain ensemble: the accepted-length /
acceleration-rate bounds (Lemma 1, Theorem 1) and the optimistic two-step update (Eq. (3))."""
import numpy as np
import pytest
from scipy.special import softmax

from oracle import oracle as O


# ------------------------------------------------- Lemma 1 / Theorem 1 ----
def test_accel_bounds_special_cases_of_the_remark():
    for T in (1, 10, 1000):
        for k in (1, 4, 9):
            for alpha in (0.0, 0.05, 0.5):
                lo, hi, glo, ghi = O.accel_bounds(0.0, T, k, alpha)
                # zero regret: every draft token accepted, the bounds meet
                assert lo == hi == (k + 1) * T
                assert ghi == pytest.approx((k + 1) / (alpha * k + 1), rel=1e-15) and glo == pytest.approx(ghi, rel=1e-14)
                # regret 2T: sqrt(Reg/(2T)) = 1, so the length bound is (k+1)T/(k+2) = Theta(T)
                lo2 = O.accel_bounds(2.0 * T, T, k, alpha)[0]
                assert lo2 == pytest.approx((k + 1) * T / (k + 2), rel=1e-14)
                # a negative regret is read as zero
                assert np.array_equal(O.accel_bounds(-3.0, T, k, alpha), O.accel_bounds(0.0, T, k, alpha))


def test_accel_bounds_gamma_is_length_over_cost():
    rng = np.random.default_rng(0)
    for _ in range(100):
        T = int(rng.integers(1, 10**6)); k = int(rng.integers(1, 20))
        alpha = float(rng.uniform(0, 1)); reg = float(rng.uniform(0, 3 * T))
        lo, hi, glo, ghi = O.accel_bounds(reg, T, k, alpha)
        cost = T * (alpha * k + 1)                      # Theorem 1's proof: gamma = E|x^| / (T (alpha k + 1))
        assert glo == pytest.approx(lo / cost, rel=1e-14) and ghi == pytest.approx(hi / cost, rel=1e-14)
        assert 0 < lo <= hi and glo <= ghi
    # monotone: more regret, weaker guarantee
    vals = [O.accel_bounds(r, 1000, 5, 0.1)[2] for r in (0, 1, 10, 100, 1000)]
    assert all(a > b for a, b in zip(vals, vals[1:]))


def test_accel_lower_bound_against_the_exact_expectation():
    """Brute force: with i.i.d. acceptance probability beta per position a step emits
    1 + beta + ... + beta^k tokens in expectation.  TV = 1 - beta, and the smallest regret
    Pinsker's inequality allows is KL = 2 TV^2 per step.  The lemma's lower bound must hold
    there for every beta and k, and becomes tight as k grows (both tend to 1/(1-beta))."""
    T = 50
    for k in (1, 2, 5, 20, 200):
        for beta in np.linspace(0.0, 1.0, 41):
            exact = T * sum(beta ** j for j in range(k + 1))
            reg = T * 2.0 * (1.0 - beta) ** 2
            lo, hi = O.accel_bounds(reg, T, k, 0.1)[:2]
            assert lo <= exact * (1 + 1e-12) and exact <= hi * (1 + 1e-12), (k, beta)
    for beta in (0.2, 0.5, 0.9):
        k = 10**7
        lo = O.accel_bounds(T * 2.0 * (1.0 - beta) ** 2, T, k, 0.1)[0]
        assert lo == pytest.approx(T / (1.0 - beta), rel=1e-5)


# ------------------------------------------------------ optimistic OGD ----
@pytest.mark.parametrize("name", ["optimistic_linear_d1.txt", "optimistic_squared_d2.txt"])
def test_optimistic_hand_computed_trajectories(golden, name):
    g = golden(name)
    d, K, T = int(g["d"]), int(g["K"]), int(g["T"])
    x = np.atleast_2d(g["x"]).reshape(T, d)
    u = np.atleast_2d(g["u"]).reshape(-1, d)
    y = None if g["loss"] == "linear" else np.atleast_1d(g["y"])
    r = O.run_optimistic(d, K, T, g["D"], [g["eta"]], g["eps"], g["loss"], x=x, y=y, u=u,
                         seg_start=np.atleast_1d(g["seg_start"]).astype(np.int64), trace=True)
    tol = 5e-7
    assert abs(r["regret"] - g["regret"]) < tol
    np.testing.assert_allclose(r["tr_f"], np.atleast_1d(g["f"]), atol=tol)
    np.testing.assert_allclose(r["tr_fu"], np.atleast_1d(g["fu"]), atol=tol)
    np.testing.assert_allclose(r["W"].ravel(), np.atleast_1d(g["W"]), atol=tol)
    np.testing.assert_allclose(r["What"].ravel(), np.atleast_1d(g["What"]), atol=tol)
    assert abs(r["delta"][0] - g["delta"]) < tol


# ------------------------------------- optimism at both levels of the ensemble ----
def test_both_levels_optimistic_hand_computed_trajectory(golden):
    g = golden("optimistic_both_levels_squared_d1.txt")
    d, K, T = int(g["d"]), int(g["K"]), int(g["T"])
    x = np.atleast_2d(g["x"]).reshape(T, d)
    r = O.run_optimistic(d, K, T, g["D"], np.atleast_1d(g["eta"]), g["eps"], g["loss"], x=x, y=np.atleast_1d(g["y"]),
                         u=np.atleast_2d(g["u"]).reshape(-1, d),
                         seg_start=np.atleast_1d(g["seg_start"]).astype(np.int64), trace=True, meta_hint=True)
    tol = 5e-7
    np.testing.assert_allclose(r["tr_p"], np.atleast_2d(g["p"]).reshape(T, K), atol=tol)
    np.testing.assert_allclose(r["tr_f"], np.atleast_1d(g["f"]), atol=tol)
    np.testing.assert_allclose(r["tr_fu"], np.atleast_1d(g["fu"]), atol=tol)
    np.testing.assert_allclose(r["W"].ravel(), np.atleast_1d(g["W"]), atol=tol)
    np.testing.assert_allclose(r["What"].ravel(), np.atleast_1d(g["What"]), atol=tol)
    np.testing.assert_allclose(r["L"], np.atleast_1d(g["L"]), atol=tol)
    np.testing.assert_allclose(r["p"], np.atleast_1d(g["p_final"]), atol=tol)
    assert abs(r["wbar"][0] - g["wbar"]) < tol and abs(r["regret"] - g["regret"]) < tol
    # and without the meta hint round 3 weighs the cumulative losses alone
    r1 = O.run_optimistic(d, K, T, g["D"], np.atleast_1d(g["eta"]), g["eps"], g["loss"], x=x, y=np.atleast_1d(g["y"]),
                          u=np.atleast_2d(g["u"]).reshape(-1, d), trace=True)
    np.testing.assert_allclose(r1["tr_p"][2], [0.8670358, 0.1329642], atol=tol)


@pytest.mark.parametrize("sparse", [False, True])
def test_meta_hint_leaves_the_base_learners_alone_and_tilts_hedge_by_the_last_loss(sparse):
    """The base learners never read the meta learner's weights, so their losses are the same with
    and without the meta hint; the hinted weights of round t are then the plain ones tilted by
    exp(-eps * last loss), and the first round is uniform.  One learner: nothing changes at all."""
    rng = np.random.default_rng(11)
    d, K, T, D, eps = 12, 4, 60, 1.0, 0.3
    eta = [0.05, 0.2, 0.8, 3.2]
    y = rng.standard_normal(T).astype(np.float32)
    u = (0.3 * rng.standard_normal((2, d))).astype(np.float32)
    seg = np.array([0, 25], np.int64)
    if sparse:
        nnz = 3
        col = np.sort(np.argsort(rng.random((T, d)), axis=1)[:, :nnz], axis=1).astype(np.int32)
        val = rng.standard_normal((T, nnz)).astype(np.float32)
        kw = dict(col=col, val=val)
    else:
        kw = dict(x=(rng.standard_normal((T, d)) / np.sqrt(d)).astype(np.float32))
    a = O.run_optimistic(d, K, T, D, eta, eps, "squared", y=y, u=u, seg_start=seg, trace=True, **kw)
    b = O.run_optimistic(d, K, T, D, eta, eps, "squared", y=y, u=u, seg_start=seg, trace=True, meta_hint=True, **kw)
    np.testing.assert_array_equal(a["tr_z"], b["tr_z"])
    np.testing.assert_array_equal(a["tr_loss"], b["tr_loss"])
    np.testing.assert_array_equal(a["W"], b["W"])
    np.testing.assert_array_equal(a["L"], b["L"])
    np.testing.assert_array_equal(b["tr_p"][0], np.full(K, 1.0 / K))
    for t in range(1, T):
        w = a["tr_p"][t] * np.exp(-eps * a["tr_loss"][t - 1])
        np.testing.assert_allclose(b["tr_p"][t], w / w.sum(), rtol=1e-12, atol=1e-15)
    w = a["p"] * np.exp(-eps * a["tr_loss"][T - 1])
    np.testing.assert_allclose(b["p"], w / w.sum(), rtol=1e-12, atol=1e-15)
    # the mixed iterate's loss follows the hinted weights
    zmix = (b["tr_p"] * b["tr_z"]).sum(axis=1)
    np.testing.assert_allclose(b["tr_f"], (zmix - y.astype(np.float64)) ** 2, rtol=1e-10, atol=1e-13)
    one = O.run_optimistic(d, 1, T, D, eta[:1], eps, "squared", y=y, u=u, seg_start=seg, **kw)
    one_h = O.run_optimistic(d, 1, T, D, eta[:1], eps, "squared", y=y, u=u, seg_start=seg, meta_hint=True, **kw)
    assert one["regret"] == one_h["regret"]
    np.testing.assert_array_equal(one["W"], one_h["W"])


def test_many_run_wrapper_with_the_meta_hint_equals_single_runs():
    from paper_2603_12617_amd import workloads as WL
    for name, over in (("c3", dict(T=150, R=3, d=24, K=3, seg_len=50)), ("c2", dict(T=120, R=3, d=10, K=3))):
        wl = WL.make(name, optimistic=2, **over)
        data = WL.generate(wl)
        ref = O.run_workload(wl, data, threads=2)
        for r in range(wl.R):
            x = data["x"] if wl.x_shared else data["x"][r]
            one = O.run_optimistic(wl.d, wl.K, wl.T, wl.D, wl.eta, wl.eps, wl.loss, x=x, y=data["y"][r], u=data["u"][r],
                                   seg_start=data["seg_start"], meta_hint=True)
            plain = O.run_optimistic(wl.d, wl.K, wl.T, wl.D, wl.eta, wl.eps, wl.loss, x=x, y=data["y"][r], u=data["u"][r],
                                     seg_start=data["seg_start"])
            assert ref["regret"][r] == one["regret"] and ref["regret"][r] != plain["regret"]
            np.testing.assert_array_equal(ref["p"][r], one["p"])
            np.testing.assert_array_equal(ref["W"][r], one["W"])


def test_optimistic_on_a_constant_gradient_is_plain_ogd_one_round_ahead():
    """Linear loss with the same gradient every round: the hint is exact from round 2 on, the
    intermediate model follows plain OGD, and the played iterate equals plain OGD's NEXT one."""
    rng = np.random.default_rng(3)
    d, T, D, eta = 5, 40, 1.0, 0.07
    g = rng.standard_normal(d).astype(np.float32)
    x = np.tile(g, (T + 1, 1))
    u = np.zeros((1, d), np.float32)
    opt = O.run_optimistic(d, 1, T, D, [eta], 0.0, "linear", x=x[:T], u=u, trace=True)
    ogd = O.run(d, 1, T + 1, D, [eta], 0.0, "linear", x=x, u=u, trace=True)
    assert opt["tr_z"][0, 0] == 0.0
    np.testing.assert_allclose(opt["tr_z"][1:, 0], ogd["tr_z"][2:, 0], rtol=0, atol=1e-14)
    short = O.run(d, 1, T, D, [eta], 0.0, "linear", x=x[:T], u=u)
    np.testing.assert_allclose(opt["What"], short["W"], rtol=0, atol=1e-14)
    assert opt["delta"][0] == pytest.approx(float(g.astype(np.float64) @ g.astype(np.float64)), rel=1e-14)


def test_optimistic_with_orthogonal_rounds_inside_the_ball_has_plain_ogd_losses():
    """x_t cycles through unit vectors: the hint step moves the played iterate only along
    x_{t-1}, orthogonal to x_t, so (no projection active) every prediction equals plain OGD's."""
    d, T = 4, 24
    x = np.zeros((T, d), np.float32)
    x[np.arange(T), np.arange(T) % d] = 1.0
    rng = np.random.default_rng(5)
    y = rng.uniform(-0.5, 0.5, T).astype(np.float32)
    u = np.zeros((1, d), np.float32)
    opt = O.run_optimistic(d, 1, T, 100.0, [0.1], 0.0, "squared", x=x, y=y, u=u, trace=True)
    ogd = O.run(d, 1, T, 100.0, [0.1], 0.0, "squared", x=x, y=y, u=u, trace=True)
    np.testing.assert_allclose(opt["tr_z"], ogd["tr_z"], rtol=0, atol=1e-14)
    assert opt["regret"] == pytest.approx(ogd["regret"], abs=1e-12)
    np.testing.assert_allclose(opt["What"], ogd["W"], rtol=0, atol=1e-14)


def _instance(rng, d, T, loss, S=3):
    x = (rng.standard_normal((T, d)) / np.sqrt(d)).astype(np.float32)
    ws = rng.standard_normal((S, d)); ws = (0.7 * ws / np.linalg.norm(ws, axis=1, keepdims=True)).astype(np.float32)
    seg_start = np.array([s * (T // S) for s in range(S)], np.int64)
    seg = np.searchsorted(seg_start, np.arange(T), side="right") - 1
    zt = np.einsum("td,td->t", x.astype(np.float64), ws[seg].astype(np.float64))
    if loss == "logistic":
        y = np.where(zt >= 0, 1.0, -1.0).astype(np.float32)
    else:
        y = (zt + 0.05 * rng.standard_normal(T)).astype(np.float32)
    return x, y, ws, seg_start, seg


@pytest.mark.parametrize("loss", ["squared", "logistic"])
def test_optimistic_regret_bound_with_explicit_constants(loss):
    """Corollary 2's proof: Reg_T <= eta delta_T + (||u_1 - w^_1||^2 + sum_t (..)) / (2 eta); on the
    radius-D ball with w^_1 = 0 that is eta delta_T + (D^2 + 4 D P_T) / (2 eta).  delta_T is
    recomputed here from the traced predictions, not taken from the reference."""
    rng = np.random.default_rng(11)
    d, T, D = 6, 300, 1.0
    for eta in (0.01, 0.1, 1.0):
        x, y, ws, seg_start, seg = _instance(rng, d, T, loss)
        r = O.run_optimistic(d, 1, T, D, [eta], 0.0, loss, x=x, y=y, u=ws, seg_start=seg_start, trace=True)
        z = r["tr_z"][:, 0]; yd = y.astype(np.float64); xd = x.astype(np.float64)
        c = 2 * (z - yd) if loss == "squared" else -yd / (1 + np.exp(yd * z))
        grads = c[:, None] * xd
        hints = np.vstack([np.zeros((1, d)), grads[:-1]])
        delta = float(((hints - grads) ** 2).sum())
        assert r["delta"][0] == pytest.approx(delta, rel=1e-12)
        P = float(np.linalg.norm(np.diff(ws[seg].astype(np.float64), axis=0), axis=1).sum())
        assert r["regret"] <= eta * delta + (D * D + 4 * D * P) / (2 * eta) + 1e-9
        assert (np.linalg.norm(r["W"], axis=1) <= D * (1 + 1e-12)).all()
        assert (np.linalg.norm(r["What"], axis=1) <= D * (1 + 1e-12)).all()


def test_optimistic_learners_are_independent_and_hedge_combines_them():
    rng = np.random.default_rng(17)
    d, T, K, D, eps = 5, 60, 3, 0.8, 0.3
    eta = [0.02, 0.2, 2.0]
    x, y, ws, seg_start, seg = _instance(rng, d, T, "squared")
    r = O.run_optimistic(d, K, T, D, eta, eps, "squared", x=x, y=y, u=ws, seg_start=seg_start, trace=True)
    for i in range(K):
        one = O.run_optimistic(d, 1, T, D, [eta[i]], 0.0, "squared", x=x, y=y, u=ws, seg_start=seg_start, trace=True)
        np.testing.assert_allclose(r["W"][i], one["W"][0], rtol=0, atol=1e-15)
        np.testing.assert_allclose(r["tr_z"][:, i], one["tr_z"][:, 0], rtol=0, atol=1e-15)
        assert r["L"][i] == pytest.approx(one["tr_loss"].sum(), rel=1e-14)
    # Hedge: weights of round t from the losses before t (library softmax), prediction = mixture
    cum = np.vstack([np.zeros((1, K)), np.cumsum(r["tr_loss"], axis=0)])
    p = softmax(-eps * cum, axis=1)
    np.testing.assert_allclose(r["tr_p"], p[:-1], rtol=0, atol=1e-14)
    np.testing.assert_allclose(r["p"], p[-1], rtol=0, atol=1e-14)
    zmix = (p[:-1] * r["tr_z"]).sum(1)
    f = (zmix - y.astype(np.float64)) ** 2
    np.testing.assert_allclose(r["tr_f"], f, rtol=0, atol=1e-13)
    assert r["regret"] == pytest.approx(float((f - r["tr_fu"]).sum()), abs=1e-11)
    np.testing.assert_allclose(r["wbar"], p[-1] @ r["W"], rtol=0, atol=1e-14)


# ------------------------------------------ optimistic OGD on sparse rounds ----
@pytest.mark.parametrize("norm_every", [0, 1, 2])
def test_sparse_optimistic_hand_computed_trajectory(golden, norm_every):
    g = golden("optimistic_sparse_squared_d3.txt")
    d, K, T = int(g["d"]), int(g["K"]), int(g["T"])
    r = O.run_optimistic(d, K, T, g["D"], [g["eta"]], g["eps"], g["loss"],
                         col=g["col"].astype(np.int32), val=g["val"], y=g["y"], u=g["u"].reshape(1, d),
                         seg_start=np.atleast_1d(g["seg_start"]).astype(np.int64), norm_every=norm_every,
                         trace=True)
    tol = 5e-7
    assert abs(r["regret"] - g["regret"]) < tol
    np.testing.assert_allclose(r["tr_f"], g["f"], atol=tol)
    np.testing.assert_allclose(r["tr_fu"], g["fu"], atol=tol)
    np.testing.assert_allclose(r["W"].ravel(), g["W"], atol=tol)
    np.testing.assert_allclose(r["What"].ravel(), g["What"], atol=tol)
    assert abs(r["delta"][0] - g["delta"]) < 5e-6


def _sparse_instance(rng, d, T, nnz, S=2, noise=0.05):
    col = np.stack([np.sort(rng.choice(d, size=nnz, replace=False)) for _ in range(T)]).astype(np.int32)
    val = (rng.standard_normal((T, nnz)) / np.sqrt(nnz)).astype(np.float32)
    x = np.zeros((T, d), np.float32)
    x[np.arange(T)[:, None], col] = val
    ws = rng.standard_normal((S, d)); ws = (0.6 * ws / np.linalg.norm(ws, axis=1, keepdims=True)).astype(np.float32)
    seg_start = np.array([s * (T // S) for s in range(S)], np.int64)
    seg = np.searchsorted(seg_start, np.arange(T), side="right") - 1
    zt = np.einsum("td,td->t", x.astype(np.float64), ws[seg].astype(np.float64))
    return col, val, x, ws, seg_start, zt


@pytest.mark.parametrize("loss", ["squared", "logistic", "linear"])
@pytest.mark.parametrize("norm_every", [0, 1, 7, 1000])
def test_sparse_optimistic_equals_its_dense_expansion(loss, norm_every):
    """The sparse form must give what the dense form of Eq. (3) gives on the same rounds written
    out as dense rows -- steps small (never projected), moderate, and far larger than the ball
    (both projections active every round); consecutive rounds share columns (d is small), so the
    hint overlaps the current row in some coordinates and not in others."""
    rng = np.random.default_rng(23 + norm_every)
    d, T, nnz, K, D, eps = 12, 90, 3, 4, 0.9, 0.2
    eta = [0.01, 0.3, 4.0, 300.0]
    col, val, x, ws, seg_start, zt = _sparse_instance(rng, d, T, nnz)
    if loss == "logistic":
        y = np.where(zt >= 0, 1.0, -1.0).astype(np.float32)
    elif loss == "squared":
        y = (zt + 0.05 * rng.standard_normal(T)).astype(np.float32)
    else:
        y = None
    assert any(len(set(col[t]) & set(col[t - 1])) not in (0, nnz) for t in range(1, T))
    dense = O.run_optimistic(d, K, T, D, eta, eps, loss, x=x, y=y, u=ws, seg_start=seg_start, trace=True)
    sp = O.run_optimistic(d, K, T, D, eta, eps, loss, col=col, val=val, y=y, u=ws, seg_start=seg_start,
                          norm_every=norm_every, trace=True)
    for k in ("W", "What", "L", "p", "wbar", "tr_z", "tr_p", "tr_loss", "tr_f", "tr_fu", "tr_zmix"):
        np.testing.assert_allclose(sp[k], dense[k], rtol=0, atol=2e-12, err_msg=k)
    np.testing.assert_allclose(sp["delta"], dense["delta"], rtol=1e-12)
    assert sp["regret"] == pytest.approx(dense["regret"], abs=1e-11)
    assert sp["max_drift"] < 1e-12
    # the projections were exercised: the large steps sit on the boundary, the small one inside
    assert np.linalg.norm(dense["What"][3]) == pytest.approx(D, rel=1e-12)
    assert np.linalg.norm(dense["What"][0]) < 0.5 * D


def test_many_run_wrappers_equal_single_runs_for_the_optimistic_update():
    """run_workload(optimistic) -- the layout arithmetic of the many-run wrapper (run strides of x,
    y and u, shared against per-run streams, dense against sparse rounds) -- against one
    run_optimistic call per run on that run's own arrays."""
    from paper_2603_12617_amd import workloads as WL
    cases = [("c3", dict(T=230, R=4, d=9, K=3, seg_len=60)),                   # shared dense stream, 4 segments
             ("c2", dict(T=150, R=3, d=7, K=4, seg_len=50)),                   # one dense stream per run
             ("c4", dict(T=120, R=3, d=11, K=2, seg_len=40)),                  # logistic
             ("c1", dict(T=100, R=3, d=5, x_shared=False)),                    # linear, per run, no labels
             ("c5", dict(T=200, R=4, d=40, K=3, nnz=4, wstar_nnz=8, seg_len=70, eta=(0.05, 1.0, 30.0)))]
    for name, over in cases:
        wl = WL.make(name, optimistic=True, **over)
        data = WL.generate(wl)
        assert data["u"].shape[1] >= 1 and wl.R >= 3
        for norm_every in ((0, 13) if wl.nnz else (0,)):
            many = O.run_workload(wl, data, norm_every=norm_every, threads=2)
            for r in range(wl.R):
                kw = dict(y=None if data["y"] is None else data["y"][r], u=data["u"][r],
                          seg_start=data["seg_start"])
                if wl.nnz:
                    kw.update(col=data["col"], val=data["val"], norm_every=norm_every)
                else:
                    kw.update(x=data["x"] if wl.x_shared else data["x"][r])
                one = O.run_optimistic(wl.d, wl.K, wl.T, wl.D, wl.eta, wl.eps, wl.loss, **kw)
                for k in ("W", "L", "p", "wbar"):
                    assert np.array_equal(many[k][r], one[k]), (name, k, r)
                assert many["regret"][r] == one["regret"]
                assert many["max_drift"][r] == one["max_drift"]
        # runs differ from each other (a wrapper that reused run 0's arrays would pass otherwise)
        assert len({float(v) for v in many["regret"]}) == wl.R
