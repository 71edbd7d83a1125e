"""Seeded synthetic round streams for the online-learner simulation.

This module only *draws data*: round inputs (features x_t, labels y_t, or
gradients g_t), the hidden parameter w* that produces the labels, and the
comparator sequence u_t that regret is measured against (Eq. (2)).  It holds
none of the learner's arithmetic (no gradient step, no projection, no Hedge
weights), so both the CPU oracle's tests and the GPU path can consume the very
same arrays without sharing any method code.

The five named workloads have the shapes and value distributions of the
benchmark configurations; they stand in for the verification-feedback losses an
LLM serving stack would hand to `Update` in Algorithm 1, which need models and
datasets that are not available here.  Every workload can be shrunk
(`make("c3", T=2000, R=4, d=200)`) for tests.

Random numbers come from numpy's counter-based Philox generator keyed by
(seed, workload id, run, stream id), so each array is independent of the order
in which the others are drawn.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np

LOSSES = ("linear", "squared", "logistic")


@dataclass(frozen=True)
class Workload:
    """Shape and hyper-parameters of one simulation (notation of Sec. 3.3 /
    Assumption 2: K base learners, domain radius D, gradient bound G)."""

    name: str
    wid: int                 # workload id, part of the RNG key
    d: int
    K: int
    T: int
    R: int
    loss: str
    D: float = 1.0
    G: float = 1.0
    x_shared: bool = True    # one x stream for all runs, or one per run
    nnz: int = 0             # 0: dense x; >0: CSR rows with exactly nnz entries
    seg_len: int = 0         # comparator redrawn every seg_len rounds (0: fixed)
    wstar_norm: float = 0.5
    wstar_nnz: int = 0       # sparse w*: number of nonzeros (0: dense)
    noise: float = 0.1
    flip: float = 0.0
    seed: int = 0
    eta: tuple = field(default=())   # filled by make()
    eps: float = 0.0
    optimistic: int = 0       # 1: Eq. (3) two-step update with the last gradient as hint; 2: the meta learner optimistic too

    @property
    def units(self) -> int:
        """Learner-updates of one full simulation: runs x K x rounds x d."""
        return self.R * self.K * self.T * self.d

    @property
    def n_seg(self) -> int:
        return 1 if self.seg_len <= 0 else (self.T + self.seg_len - 1) // self.seg_len


def step_grid(D: float, G: float, T: int, K: int) -> tuple:
    """Geometric grid eta_i = 2^i D/(G sqrt(T)), i = 0..K-1 (the grid in the
    proof of Corollary 3, with its index i-1 written as i)."""
    base = D / (G * math.sqrt(T))
    return tuple(base * (2.0 ** i) for i in range(K))


def paper_N(T: int) -> int:
    """Number of base learners the proof of Corollary 3 prescribes."""
    return math.ceil(0.5 * math.log2(1 + T)) + 1


def meta_rate(K: int, T: int) -> float:
    return math.sqrt(math.log(K) / T) if K > 1 else 0.0


_BASE: Dict[str, Workload] = {
    "c1": Workload("c1", 1, d=10, K=1, T=1000, R=1, loss="linear"),
    "c2": Workload("c2", 2, d=100, K=15, T=10000, R=64, loss="squared", x_shared=False),
    "c3": Workload("c3", 3, d=1000, K=17, T=100000, R=256, loss="squared",
                   seg_len=1000, wstar_norm=0.8),
    "c4": Workload("c4", 4, d=4096, K=16, T=20000, R=1024, loss="logistic",
                   wstar_norm=1.0, flip=0.1),
    "c5": Workload("c5", 5, d=1 << 20, K=8, T=100000, R=16, loss="squared",
                   nnz=32, wstar_nnz=1024),
}


def make(name: str, **over) -> Workload:
    """Named workload, optionally with fields overridden; the step grid and the
    meta rate follow the (possibly overridden) D, G, T, K unless given."""
    wl = replace(_BASE[name], **{k: v for k, v in over.items() if k not in ("eta", "eps")})
    eta = tuple(over["eta"]) if "eta" in over else step_grid(wl.D, wl.G, wl.T, wl.K)
    eps = over["eps"] if "eps" in over else meta_rate(wl.K, wl.T)
    if len(eta) != wl.K:
        raise ValueError("eta must have K entries")
    if wl.wstar_nnz > wl.d:
        wl = replace(wl, wstar_nnz=wl.d)
    return replace(wl, eta=eta, eps=eps)


def names() -> List[str]:
    return list(_BASE)


def _rng(wl: Workload, run: int, stream: int) -> np.random.Generator:
    k0 = ((wl.seed & 0xFFFFFFFF) << 32) | ((wl.wid & 0xFFFF) << 16) | (stream & 0xFFFF)
    return np.random.Generator(np.random.Philox(key=[k0, run & 0xFFFFFFFFFFFFFFFF]))


_S_X, _S_W, _S_NOISE, _S_FLIP, _S_COL, _S_VAL, _S_SUPP = range(7)


def _unit_rows(rng: np.random.Generator, n: int, d: int) -> np.ndarray:
    """n directions uniform on the unit sphere of R^d (float64)."""
    v = rng.standard_normal((n, d))
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    return v


def _csr_rows(wl: Workload) -> tuple:
    """T rows of exactly nnz distinct column indices, ascending, with values
    N(0, 1/nnz)."""
    rng = _rng(wl, 0, _S_COL)
    if wl.nnz > wl.d:
        raise ValueError("a sparse row cannot have more entries than columns")
    if wl.nnz * 8 > wl.d:       # rows that fill much of the width: a random subset (redrawing would not end)
        col = np.sort(np.argsort(rng.random((wl.T, wl.d)), axis=1)[:, :wl.nnz], axis=1).astype(np.int64)
    else:
        col = np.sort(rng.integers(0, wl.d, size=(wl.T, wl.nnz), dtype=np.int64), axis=1)
    while True:
        bad = np.nonzero((col[:, 1:] == col[:, :-1]).any(axis=1))[0]
        if bad.size == 0:
            break
        col[bad] = np.sort(rng.integers(0, wl.d, size=(bad.size, wl.nnz), dtype=np.int64), axis=1)
    val = _rng(wl, 0, _S_VAL).standard_normal((wl.T, wl.nnz), dtype=np.float32)
    val *= np.float32(1.0 / math.sqrt(wl.nnz))
    return col.astype(np.int32), val


def generate(wl: Workload) -> Dict[str, Optional[np.ndarray]]:
    """Draw every array of a workload.

    Returns a dict with
      x    float32 [T][d] (shared) or [R][T][d] (per run); for the linear loss
           this is the gradient stream g_t; None when sparse
      col  int32 [T][nnz], val float32 [T][nnz]   (sparse only, shared by runs)
      y    float32 [R][T]; None for the linear loss
      u    float32 [R][S][d] comparator segments, seg_start int64 [S]
    """
    if wl.loss not in LOSSES:
        raise ValueError(wl.loss)
    out: Dict[str, Optional[np.ndarray]] = {"x": None, "col": None, "val": None, "y": None}
    S = wl.n_seg
    seg_start = np.arange(S, dtype=np.int64) * max(wl.seg_len, 0)
    out["seg_start"] = seg_start

    if wl.loss == "linear":
        # g_t ~ N(0, I) rescaled to norm G in double, stored in float32.  The
        # comparator is the best fixed point of the ball in hindsight for the
        # stored stream: u* = -D S/||S||, S = sum_t g_t.
        shape = (wl.T, wl.d) if wl.x_shared else (wl.R, wl.T, wl.d)
        g = _rng(wl, 0, _S_X).standard_normal(shape)
        g *= wl.G / np.linalg.norm(g, axis=-1, keepdims=True)
        g32 = g.astype(np.float32)
        out["x"] = g32
        tot = g32.astype(np.float64).sum(axis=-2)          # [d] or [R][d]
        tot = np.broadcast_to(tot, (wl.R, wl.d)) if wl.x_shared else tot
        nrm = np.linalg.norm(tot, axis=1, keepdims=True)
        u = np.where(nrm > 0, -wl.D * tot / np.where(nrm > 0, nrm, 1.0), 0.0)
        out["u"] = np.ascontiguousarray(u[:, None, :].astype(np.float32))
        return out

    # hidden parameters: one per (run, segment)
    u = np.zeros((wl.R, S, wl.d), dtype=np.float32)
    for r in range(wl.R):
        rw = _rng(wl, r, _S_W)
        if wl.wstar_nnz and wl.wstar_nnz < wl.d:
            for s in range(S):
                supp = _rng(wl, r * S + s, _S_SUPP).choice(wl.d, size=wl.wstar_nnz, replace=False)
                v = rw.standard_normal(wl.wstar_nnz)
                v *= wl.wstar_norm / np.linalg.norm(v)
                u[r, s, supp] = v.astype(np.float32)
        else:
            u[r] = (wl.wstar_norm * _unit_rows(rw, S, wl.d)).astype(np.float32)
    out["u"] = u

    # round inputs and the clean responses <w*, x_t>
    if wl.nnz:
        col, val = _csr_rows(wl)
        out["col"], out["val"] = col, val
        clean = np.empty((wl.R, wl.T), dtype=np.float64)
        for r in range(wl.R):
            for s in range(S):
                a, b = int(seg_start[s]), int(seg_start[s + 1]) if s + 1 < S else wl.T
                clean[r, a:b] = (u[r, s][col[a:b]].astype(np.float64) * val[a:b]).sum(axis=1)
    else:
        sig = np.float32(1.0 / math.sqrt(wl.d))
        if wl.x_shared:
            x = _rng(wl, 0, _S_X).standard_normal((wl.T, wl.d), dtype=np.float32)
            x *= sig
        else:
            x = np.empty((wl.R, wl.T, wl.d), dtype=np.float32)
            for r in range(wl.R):
                x[r] = _rng(wl, r, _S_X).standard_normal((wl.T, wl.d), dtype=np.float32)
            x *= sig
        out["x"] = x
        clean = np.empty((wl.R, wl.T), dtype=np.float32)
        for s in range(S):
            a, b = int(seg_start[s]), int(seg_start[s + 1]) if s + 1 < S else wl.T
            if wl.x_shared:
                clean[:, a:b] = u[:, s, :] @ x[a:b].T
            else:
                clean[:, a:b] = np.einsum("rd,rtd->rt", u[:, s, :], x[:, a:b])

    y = np.empty((wl.R, wl.T), dtype=np.float32)
    for r in range(wl.R):
        if wl.loss == "squared":
            y[r] = clean[r] + wl.noise * _rng(wl, r, _S_NOISE).standard_normal(wl.T)
        else:  # logistic: labels in {-1,+1}, sign(0) = +1, flipped with prob. `flip`
            lab = np.where(clean[r] >= 0, 1.0, -1.0)
            flips = _rng(wl, r, _S_FLIP).random(wl.T) < wl.flip
            y[r] = np.where(flips, -lab, lab)
    out["y"] = y
    return out


def run_slice(wl: Workload, data: Dict[str, Optional[np.ndarray]], runs) -> tuple:
    """Restrict a workload and its arrays to a subset of runs (for checking a
    few runs of a large simulation against the oracle)."""
    runs = np.asarray(runs, dtype=np.int64)
    sub = dict(data)
    if data["y"] is not None:
        sub["y"] = np.ascontiguousarray(data["y"][runs])
    sub["u"] = np.ascontiguousarray(data["u"][runs])
    if data["x"] is not None and not wl.x_shared:
        sub["x"] = np.ascontiguousarray(data["x"][runs])
    return replace(wl, R=int(runs.size)), sub


# ---------------------------------------------------------------------------
# Synthetic draft / target distributions for the verification step of Algorithm 1
# (stand-ins for the token distributions of a draft and a target LLM; no method
# arithmetic here: logits, softmax, and the draws the method consumes as inputs).
SPECDEC = {
    "v1": dict(B=96, k=4, V=1000),        # small: the CPU reference finishes in seconds
    "v2": dict(B=1024, k=4, V=32000),     # Llama-2 / Vicuna vocabulary
    "v3": dict(B=256, k=4, V=151936),     # Qwen3 vocabulary
}


def specdec_inputs(B: int, k: int, V: int, seed: int = 0, sharp: float = 2.5, noise: float = 0.6,
                   exact_frac: float = 0.0):
    """Returns dict(p [B][k+1][V] f32, q [B][k][V] f32, tok [B][k] i32, r [B][k] f32, u [B] u32).
    Target logits are sharp * N(0,1) (a few dominant tokens, a long tail); the draft's are the
    target's plus noise * N(0,1); a fraction exact_frac of the draft rows equals the target row
    (always accepted).  tok[b][j] is drawn from q[b][j]."""
    rng = np.random.Generator(np.random.Philox(key=[(seed & 0xFFFFFFFF) << 32 | 0x5D, B * 1000003 + k * 1009 + V]))
    p = np.empty((B, k + 1, V), np.float32)
    q = np.empty((B, k, V), np.float32)
    tok = np.empty((B, k), np.int32)
    step = max(1, (1 << 24) // ((k + 1) * V))
    for b0 in range(0, B, step):
        b1 = min(B, b0 + step)
        lp = sharp * rng.standard_normal((b1 - b0, k + 1, V))
        lq = lp[:, :k] + noise * rng.standard_normal((b1 - b0, k, V))
        same = rng.random((b1 - b0, k)) < exact_frac
        lq[same] = lp[:, :k][same]
        pp = np.exp(lp - lp.max(axis=2, keepdims=True)); pp /= pp.sum(axis=2, keepdims=True)
        qq = np.exp(lq - lq.max(axis=2, keepdims=True)); qq /= qq.sum(axis=2, keepdims=True)
        p[b0:b1] = pp
        q[b0:b1] = qq
        cdf = np.cumsum(qq, axis=2)
        draw = rng.random((b1 - b0, k, 1)) * cdf[:, :, -1:]
        tok[b0:b1] = np.minimum((cdf < draw).sum(axis=2), V - 1)
    r = rng.random((B, k), dtype=np.float32)
    u = rng.integers(0, 1 << 32, size=B, dtype=np.uint64).astype(np.uint32)
    return dict(p=p, q=q, tok=tok, r=r, u=u)
