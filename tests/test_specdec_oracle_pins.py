"""Pins for the CPU reference of the verification step of Algorithm 1: what speculative
sampling guarantees mathematically, checked without using the reference to produce the
expectation."""
import numpy as np
import pytest

from oracle import specdec_oracle as SO
from paper_2603_12617_amd import workloads as WL


def _softmax(l):
    e = np.exp(l - l.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def test_acceptance_is_one_minus_total_variation():
    rng = np.random.default_rng(0)
    p = _softmax(2 * rng.standard_normal((5, 4, 300))).astype(np.float32)
    q = _softmax(2 * rng.standard_normal((5, 3, 300))).astype(np.float32)
    acc = SO.acceptance(p, q)
    tv = 0.5 * np.abs(p[:, :3].astype(np.float64) - q.astype(np.float64)).sum(axis=2)
    mass = 0.5 * (p[:, :3].astype(np.float64).sum(2) + q.astype(np.float64).sum(2))   # = 1 up to float32 rounding
    np.testing.assert_allclose(acc, mass - tv, rtol=0, atol=1e-12)
    same = SO.acceptance(p[:, :4], p[:, :3])
    np.testing.assert_allclose(same, p[:, :3].astype(np.float64).sum(2), atol=1e-12)


def test_hand_worked_step():
    """V = 4, k = 2.  Position 0: x = 1, q(1) = 0.5, p(1) = 0.25: ratio 0.5; r = 0.4 accepts.
    Position 1: x = 0, q(0) = 0.5, p(0) = 0.125: ratio 0.25; r = 0.3 rejects -> n = 1.
    Residual at position 1: max(0, p - q) = (0, 0.125, 0.25, 0) -> p' = (0, 1/3, 2/3, 0):
    u/2^32 < 1/3 gives token 1, otherwise token 2."""
    p = np.array([[[0.25, 0.25, 0.25, 0.25], [0.125, 0.25, 0.5, 0.125], [0.25, 0.25, 0.25, 0.25]]], np.float32)
    q = np.array([[[0.25, 0.5, 0.125, 0.125], [0.5, 0.125, 0.25, 0.125]]], np.float32)
    tok = np.array([[1, 0]], np.int32)
    cases = (((0.4, 0.3), 0.2, (1, 1)), ((0.4, 0.3), 0.5, (1, 2)),
             # r_0 = 0.6 > 0.5 rejects at once; max(0, p_0 - q_0) = (0, 0, .125, .125): u = 0.1 -> token 2
             ((0.6, 0.3), 0.1, (0, 2)),
             # both accepted (r_1 q = 0.125 <= p = 0.125 is the boundary): next from the uniform p_2
             ((0.4, 0.2), 0.6, (2, 2)), ((0.4, 0.25), 0.9, (2, 3)))
    for rr, uu, want in cases:
        n, nx = SO.verify(p, q, tok, np.array([rr], np.float32), np.array([int(uu * 2 ** 32)], np.uint32))
        assert (n[0], nx[0]) == want, (rr, uu)


def test_inverse_cdf_splits_the_unit_interval_in_proportion_to_the_residual():
    rng = np.random.default_rng(1)
    V = 7
    p = _softmax(rng.standard_normal((1, 2, V))).astype(np.float32)
    q = _softmax(rng.standard_normal((1, 1, V))).astype(np.float32)
    tok = np.array([[int(np.argmax(q[0, 0] - p[0, 0]))]], np.int32)      # a token with p < q
    r = np.array([[0.999999]], np.float32)                                # rejected
    assert r[0, 0] * q[0, 0, tok[0, 0]] > p[0, 0, tok[0, 0]]
    N = 20000
    us = (np.arange(N, dtype=np.float64) + 0.5) / N
    counts = np.zeros(V)
    for uu in us:
        n, nx = SO.verify(p, q, tok, r, np.array([int(uu * 2 ** 32)], np.uint32))
        assert n[0] == 0
        counts[nx[0]] += 1
    m = np.maximum(0.0, p[0, 0].astype(np.float64) - q[0, 0].astype(np.float64))
    np.testing.assert_allclose(counts / N, m / m.sum(), atol=2.0 / N + 1e-7)
    # monotone in u, and tokens with p <= q are never drawn
    assert (counts[m == 0] == 0).all()


def test_emitted_token_follows_the_target_distribution():
    """The theorem behind speculative sampling: whatever the draft, the first emitted token of a
    step is distributed as the target p.  Monte Carlo with k = 1 over a small vocabulary."""
    rng = np.random.default_rng(2)
    V, N = 6, 200000
    p1 = _softmax(1.5 * rng.standard_normal(V)); q1 = _softmax(1.5 * rng.standard_normal(V))
    p = np.broadcast_to(np.stack([p1, p1])[None], (N, 2, V)).astype(np.float32).copy()
    q = np.broadcast_to(q1[None, None], (N, 1, V)).astype(np.float32).copy()
    tok = rng.choice(V, size=(N, 1), p=q1).astype(np.int32)
    r = rng.random((N, 1), dtype=np.float32)
    u = rng.integers(0, 1 << 32, size=N, dtype=np.uint64).astype(np.uint32)
    n, nx = SO.verify(p, q, tok, r, u)
    first = np.where(n == 1, tok[:, 0], nx)          # accepted draft token, else the resampled one
    freq = np.bincount(first, minlength=V) / N
    sigma = np.sqrt(p1 * (1 - p1) / N)
    assert (np.abs(freq - p1) < 5 * sigma + 1e-4).all(), (freq, p1)
    # acceptance frequency is Eq. (1)
    acc = float(SO.acceptance(p[:1], q[:1])[0, 0])
    assert abs((n == 1).mean() - acc) < 5 * np.sqrt(acc * (1 - acc) / N)


def test_expected_tokens_per_step_with_iid_positions():
    """With the same (p, q) at every position, E[n + 1] = (1 - Acc^(k+1)) / (1 - Acc) (the
    expression the proof of Lemma 1 starts from)."""
    rng = np.random.default_rng(3)
    V, k, N = 5, 4, 100000
    p1 = _softmax(rng.standard_normal(V)); q1 = _softmax(rng.standard_normal(V))
    p = np.broadcast_to(p1[None, None], (N, k + 1, V)).astype(np.float32).copy()
    q = np.broadcast_to(q1[None, None], (N, k, V)).astype(np.float32).copy()
    tok = rng.choice(V, size=(N, k), p=q1).astype(np.int32)
    r = rng.random((N, k), dtype=np.float32)
    u = rng.integers(0, 1 << 32, size=N, dtype=np.uint64).astype(np.uint32)
    n, nx = SO.verify(p, q, tok, r, u)
    acc = float(np.minimum(p1, q1).sum())
    want = (1 - acc ** (k + 1)) / (1 - acc)
    got = (n + 1).mean()
    assert abs(got - want) < 5 * (n + 1).std() / np.sqrt(N), (got, want)
    # n is geometric: P(n >= j) = Acc^j
    for j in range(1, k + 1):
        pj = acc ** j
        assert abs((n >= j).mean() - pj) < 5 * np.sqrt(pj * (1 - pj) / N) + 1e-4


def test_edge_cases():
    V, k = 8, 3
    rng = np.random.default_rng(4)
    p = _softmax(rng.standard_normal((1, k + 1, V))).astype(np.float32)
    q = p[:, :k].copy()
    tok = np.array([[2, 5, 7]], np.int32)
    # identical distributions: every token accepted for any r < 1; next drawn from p_k
    n, nx = SO.verify(p, q, tok, np.full((1, k), 0.9999999, np.float32), np.array([0], np.uint32))
    assert n[0] == k and nx[0] == int(np.nonzero(p[0, k] >= 2.0 ** -40)[0][0])
    n, nx = SO.verify(p, q, tok, np.zeros((1, k), np.float32), np.array([2 ** 32 - 1], np.uint32))
    assert n[0] == k and nx[0] == V - 1 or p[0, k, V - 1] * 2 ** 32 < 1
    # q(x_j) = 0 accepts (r * 0 <= p)
    q2 = q.copy(); q2[0, 0, 2] = 0.0
    assert SO.verify(p, q2, tok, np.full((1, k), 0.5, np.float32), np.array([7], np.uint32))[0][0] == k
    # p(x_0) = 0 < r q(x_0) rejects at once; the residual never returns x_0
    p3 = p.copy(); p3[0, 0, 2] = 0.0
    n, nx = SO.verify(p3, q, tok, np.full((1, k), 0.5, np.float32), np.array([123456789], np.uint32))
    assert n[0] == 0 and nx[0] != 2
    # out-of-range draft tokens are clamped, not read out of bounds
    SO.verify(p, q, np.array([[-5, 99, 3]], np.int32), np.full((1, k), 0.5, np.float32), np.array([1], np.uint32))


def test_generated_inputs_are_distributions_and_tokens_follow_the_draft():
    d = WL.specdec_inputs(B=64, k=3, V=50, seed=5)
    assert d["p"].shape == (64, 4, 50) and d["q"].shape == (64, 3, 50)
    np.testing.assert_allclose(d["p"].astype(np.float64).sum(2), 1.0, atol=1e-5)
    np.testing.assert_allclose(d["q"].astype(np.float64).sum(2), 1.0, atol=1e-5)
    assert d["tok"].min() >= 0 and d["tok"].max() < 50 and (d["r"] >= 0).all() and (d["r"] < 1).all()
    e = WL.specdec_inputs(B=64, k=3, V=50, seed=5)
    assert all(np.array_equal(d[k], e[k]) for k in d)
    # drafts drawn from q: the mean probability of the drawn token is sum q^2
    big = WL.specdec_inputs(B=4000, k=1, V=20, seed=6)
    qq = big["q"][:, 0].astype(np.float64)
    drawn = qq[np.arange(4000), big["tok"][:, 0]].mean()
    assert abs(drawn - (qq ** 2).sum(1).mean()) < 0.02
