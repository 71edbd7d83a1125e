"""Plain CPU reference of the verification step of speculative decoding -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the bench's reported CPU baseline may import this module; it
shares no code with the GPU library.

Follows Algorithm 1 step by step for one batch of independent steps:
  accepted length  n = min({j : r_j > p_j(x_j)/q_j(x_j)} U {k})   (0-based j), the test taken
                   as NOT(r_j * q_j(x_j) <= p_j(x_j)) in float32 (the precision the decision is
                   defined in; a draft token with q = 0 is accepted);
  residual         p'(x) proportional to max(0, p_n(x) - q_n(x)) if n < k, else p' = p_k;
  next token       inverse CDF of p' with the given uniform.
The draw is defined in exact integer arithmetic (so that no summation order can change it):
m(x) = trunc(2^40 max(0, p_n(x) - q_n(x))), the difference in float32; Z = sum m;
target = floor(Z u / 2^32) with u a uniform 32-bit integer; next = min{x : sum_{x'<=x} m(x') >
target}.  If Z == 0, p' = p_n.  Readings: Algorithm 1 leaves the sampler of p' open; the
resolution 2^-40 drops at most V 2^-40 of probability mass.

acceptance() is Eq. (1) written out: sum_x min(p(x), q(x)) in float64.
"""
import numpy as np

FIXED_BITS = 40


def _fixed(m32: np.ndarray) -> np.ndarray:
    # m32 is float32; scaling by a power of two is exact, the cast truncates
    return np.floor(m32.astype(np.float64) * float(1 << FIXED_BITS)).astype(np.uint64)


def verify(p, q, tok, r, u):
    """p [B][k+1][V] f32, q [B][k][V] f32, tok [B][k] i32, r [B][k] f32, u [B] u32 ->
    (n [B] i32, next [B] i32)."""
    p = np.asarray(p, np.float32); q = np.asarray(q, np.float32)
    tok = np.asarray(tok); r = np.asarray(r, np.float32); u = np.asarray(u, np.uint32)
    B, k, V = q.shape
    assert p.shape == (B, k + 1, V) and tok.shape == (B, k) and r.shape == (B, k) and u.shape == (B,)
    n_out = np.empty(B, np.int32); nx_out = np.empty(B, np.int32)
    for b in range(B):
        n = k
        for j in range(k):
            t = min(max(int(tok[b, j]), 0), V - 1)
            lhs = np.float32(r[b, j]) * np.float32(q[b, j, t])        # one float32 rounding
            if not (lhs <= p[b, j, t]):
                n = j
                break
        if n < k:
            m = _fixed(np.maximum(np.float32(0), p[b, n] - q[b, n]))
            if int(m.sum(dtype=np.uint64)) == 0:
                m = _fixed(p[b, n])
        else:
            m = _fixed(p[b, k])
        prefix = np.cumsum(m, dtype=np.uint64)
        Z = int(prefix[-1])
        if Z == 0:
            nx = 0
        else:
            target = (Z * int(u[b])) >> 32
            nx = int(np.searchsorted(prefix, np.uint64(target), side="right"))
        n_out[b] = n
        nx_out[b] = nx
    return n_out, nx_out


def acceptance(p, q):
    """acc[b][j] = sum_x min(p_j(x), q_j(x))  (Eq. (1); = 1 - TV(p_j, q_j))."""
    p = np.asarray(p, np.float32); q = np.asarray(q, np.float32)
    k = q.shape[1]
    return np.minimum(p[:, :k].astype(np.float64), q.astype(np.float64)).sum(axis=2)
