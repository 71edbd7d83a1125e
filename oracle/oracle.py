"""ctypes front end of the double-precision C reference -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the bench's reported CPU baseline may import
this module; the GPU library never does, and nothing here imports the GPU
binding.  The arithmetic lives in oco_oracle.c; this file only marshals numpy
arrays.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np

from . import build as _build

LOSS_ID = {"linear": 0, "squared": 1, "logistic": 2}

_lib = None


class _Trace(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("p", "z", "loss", "g2", "f", "fu", "zmix", "wnorm")]


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) else _build.build()
        _lib = C.CDLL(path)
        d = C.c_double
        _lib.oco_oracle_loss.restype = d
        _lib.oco_oracle_loss.argtypes = [C.c_int, d, d]
        _lib.oco_oracle_slope.restype = d
        _lib.oco_oracle_slope.argtypes = [C.c_int, d, d]
        _lib.oco_oracle_project.restype = None
        _lib.oco_oracle_project.argtypes = [C.c_void_p, C.c_int64, d]
        _lib.oco_oracle_hedge.restype = None
        _lib.oco_oracle_hedge.argtypes = [C.c_void_p, C.c_int64, d, C.c_void_p]
        _lib.oco_oracle_run.restype = C.c_int
        _lib.oco_oracle_run.argtypes = (
            [C.c_int64, C.c_int64, C.c_int64, d, C.c_void_p, d, C.c_int]
            + [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64]
            + [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64]
            + [C.c_void_p] * 5 + [C.c_void_p, C.c_void_p])
        _lib.oco_oracle_run_many.restype = C.c_int
        _lib.oco_oracle_run_many.argtypes = (
            [C.c_int64] * 4 + [d, C.c_void_p, d, C.c_int, C.c_int]
            + [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64]
            + [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int]
            + [C.c_void_p] * 5 + [C.c_void_p, C.c_void_p])
        _lib.oco_oracle_accel_bounds.restype = None
        _lib.oco_oracle_accel_bounds.argtypes = [d, C.c_int64, C.c_int64, d, C.c_void_p]
        _lib.oco_oracle_run_optimistic.restype = C.c_int
        _lib.oco_oracle_run_optimistic.argtypes = (
            [C.c_int64, C.c_int64, C.c_int64, d, C.c_void_p, d, C.c_int]
            + [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64]
            + [C.c_void_p] * 7 + [C.c_void_p])
        _lib.oco_oracle_run_optimistic_sparse.restype = C.c_int
        _lib.oco_oracle_run_optimistic_sparse.argtypes = (
            [C.c_int64, C.c_int64, C.c_int64, d, C.c_void_p, d, C.c_int]
            + [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64]
            + [C.c_void_p] * 8 + [C.c_void_p])
        _lib.oco_oracle_run_many_optimistic.restype = C.c_int
        _lib.oco_oracle_run_many_optimistic.argtypes = (
            [C.c_int64] * 4 + [d, C.c_void_p, d, C.c_int, C.c_int]
            + [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64]
            + [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int]
            + [C.c_void_p] * 5 + [C.c_void_p, C.c_void_p])
        # the same three with the meta learner's hint as a last argument
        for name in ("oco_oracle_run_optimistic", "oco_oracle_run_optimistic_sparse", "oco_oracle_run_many_optimistic"):
            f = getattr(_lib, name + "_meta")
            f.restype = C.c_int
            f.argtypes = list(getattr(_lib, name).argtypes) + [C.c_int]
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def loss(kind: str, z: float, y: float) -> float:
    return lib().oco_oracle_loss(LOSS_ID[kind], float(z), float(y))


def slope(kind: str, z: float, y: float) -> float:
    return lib().oco_oracle_slope(LOSS_ID[kind], float(z), float(y))


def project(v, D: float) -> np.ndarray:
    out = np.array(v, dtype=np.float64).reshape(-1).copy()
    lib().oco_oracle_project(_ptr(out), out.size, float(D))
    return out


def hedge(L, eps: float) -> np.ndarray:
    L = np.ascontiguousarray(L, dtype=np.float64)
    p = np.empty_like(L)
    lib().oco_oracle_hedge(_ptr(L), L.size, float(eps), _ptr(p))
    return p


def run(d: int, K: int, T: int, D: float, eta, eps: float, loss: str, *,
        x=None, col=None, val=None, y=None, u=None, seg_start=None,
        norm_every: int = 0, trace: bool = False) -> Dict[str, np.ndarray]:
    """One run of the learner; arrays are for that run only:
    x [T][d] (or col/val [T][nnz]), y [T], u [S][d], seg_start [S]."""
    eta = np.ascontiguousarray(eta, dtype=np.float64)
    assert eta.size == K
    x, val, y, u = _f32(x), _f32(val), _f32(y), _f32(u)
    col = None if col is None else np.ascontiguousarray(col, dtype=np.int32)
    nnz = 0 if col is None else col.shape[1]
    u = u.reshape(-1, d)
    S = u.shape[0]
    seg_start = (np.zeros(1, np.int64) if seg_start is None
                 else np.ascontiguousarray(seg_start, dtype=np.int64))
    assert seg_start.size == S
    if x is not None:
        assert x.shape == (T, d)
    if col is not None:
        assert col.shape == (T, nnz) and val.shape == (T, nnz)
    if y is not None:
        assert y.shape == (T,)
    W = np.empty((K, d)); L = np.empty(K); p = np.empty(K); wbar = np.empty(d)
    reg = np.zeros(1); drift = np.zeros(1)
    tr = None
    res: Dict[str, np.ndarray] = {}
    if trace:
        tr = _Trace()
        for name, shape in (("p", (T, K)), ("z", (T, K)), ("loss", (T, K)), ("g2", (T, K)),
                            ("f", (T,)), ("fu", (T,)), ("zmix", (T,)), ("wnorm", (T, K))):
            arr = np.zeros(shape)
            res["tr_" + name] = arr
            setattr(tr, name, arr.ctypes.data)
    rc = lib().oco_oracle_run(d, K, T, float(D), _ptr(eta), float(eps), LOSS_ID[loss],
                              _ptr(x), _ptr(col), _ptr(val), nnz, _ptr(y), _ptr(u),
                              _ptr(seg_start), S, int(norm_every),
                              _ptr(W), _ptr(L), _ptr(p), _ptr(wbar), _ptr(reg), _ptr(drift),
                              C.byref(tr) if tr is not None else None)
    if rc != 0:
        raise ValueError("oco_oracle_run rejected its arguments")
    res.update(W=W, L=L, p=p, wbar=wbar, regret=float(reg[0]), max_drift=float(drift[0]))
    return res


def accel_bounds(reg: float, T: int, k: int, alpha: float) -> np.ndarray:
    """[len_lo, len_hi, gamma_lo, gamma_hi] of Lemma 1 / Theorem 1."""
    out = np.empty(4)
    lib().oco_oracle_accel_bounds(float(reg), int(T), int(k), float(alpha), _ptr(out))
    return out


def run_optimistic(d: int, K: int, T: int, D: float, eta, eps: float, loss: str, *,
                   x=None, col=None, val=None, y=None, u=None, seg_start=None, norm_every: int = 0,
                   trace: bool = False, meta_hint: bool = False) -> Dict[str, np.ndarray]:
    """One run of K optimistic learners (Eq. (3), last-gradient hint) on a dense stream x [T][d]
    or on sparse rounds col/val [T][nnz].  meta_hint: the meta learner is optimistic as well
    (Hedge on L_{t-1} + the last observed loss; appendix on combining optimism and ensemble)."""
    eta = np.ascontiguousarray(eta, dtype=np.float64)
    assert eta.size == K
    x, val, y, u = _f32(x), _f32(val), _f32(y), _f32(u)
    col = None if col is None else np.ascontiguousarray(col, dtype=np.int32)
    u = u.reshape(-1, d)
    S = u.shape[0]
    seg_start = (np.zeros(1, np.int64) if seg_start is None
                 else np.ascontiguousarray(seg_start, dtype=np.int64))
    assert seg_start.size == S
    assert (x is None) != (col is None)
    if x is not None:
        assert x.shape == (T, d)
    else:
        assert col.shape == val.shape and col.shape[0] == T
    W = np.empty((K, d)); What = np.empty((K, d)); L = np.empty(K); p = np.empty(K); wbar = np.empty(d)
    reg = np.zeros(1); delta = np.zeros(K); drift = np.zeros(1)
    tr = None
    res: Dict[str, np.ndarray] = {}
    if trace:
        tr = _Trace()
        for name, shape in (("p", (T, K)), ("z", (T, K)), ("loss", (T, K)),
                            ("f", (T,)), ("fu", (T,)), ("zmix", (T,))):
            arr = np.zeros(shape)
            res["tr_" + name] = arr
            setattr(tr, name, arr.ctypes.data)
    if col is not None:
        rc = lib().oco_oracle_run_optimistic_sparse_meta(
            d, K, T, float(D), _ptr(eta), float(eps), LOSS_ID[loss], _ptr(col), _ptr(val), col.shape[1],
            _ptr(y), _ptr(u), _ptr(seg_start), S, int(norm_every),
            _ptr(W), _ptr(What), _ptr(L), _ptr(p), _ptr(wbar), _ptr(reg), _ptr(delta), _ptr(drift),
            C.byref(tr) if tr is not None else None, int(bool(meta_hint)))
    else:
        rc = lib().oco_oracle_run_optimistic_meta(d, K, T, float(D), _ptr(eta), float(eps), LOSS_ID[loss],
                                                  _ptr(x), _ptr(y), _ptr(u), _ptr(seg_start), S,
                                                  _ptr(W), _ptr(What), _ptr(L), _ptr(p), _ptr(wbar), _ptr(reg),
                                                  _ptr(delta), C.byref(tr) if tr is not None else None,
                                                  int(bool(meta_hint)))
    if rc != 0:
        raise ValueError("oco_oracle_run_optimistic rejected its arguments")
    res.update(W=W, What=What, L=L, p=p, wbar=wbar, regret=float(reg[0]), delta=delta,
               max_drift=float(drift[0]))
    return res


def run_workload(wl, data, *, threads: int = 0, norm_every: Optional[int] = None):
    """All R runs of a workload (fields as in paper_2603_12617_amd.workloads:
    any object with d, K, T, R, D, eta, eps, loss, x_shared, nnz), one run per
    OpenMP thread.  Returns W[R][K][d], L, p, wbar, regret[R], threads."""
    R, K, d, T = wl.R, wl.K, wl.d, wl.T
    eta = np.ascontiguousarray(wl.eta, dtype=np.float64)
    x, val, y, u = _f32(data.get("x")), _f32(data.get("val")), _f32(data.get("y")), _f32(data["u"])
    col = data.get("col")
    col = None if col is None else np.ascontiguousarray(col, dtype=np.int32)
    nnz = 0 if col is None else col.shape[1]
    seg_start = np.ascontiguousarray(data["seg_start"], dtype=np.int64)
    S = seg_start.size
    assert u.shape == (R, S, d)
    if norm_every is None:
        norm_every = 1000 if nnz else 0
    W = np.empty((R, K, d)); L = np.empty((R, K)); p = np.empty((R, K)); wbar = np.empty((R, d))
    reg = np.zeros(R); drift = np.zeros(R); used = C.c_int(0)
    if getattr(wl, "optimistic", False):
        bad = lib().oco_oracle_run_many_optimistic_meta(R, d, K, T, float(wl.D), _ptr(eta), float(wl.eps),
                                                        LOSS_ID[wl.loss], int(bool(wl.x_shared)),
                                                        _ptr(x), _ptr(col), _ptr(val), nnz,
                                                        _ptr(y), _ptr(u), _ptr(seg_start), S,
                                                        int(norm_every), int(threads),
                                                        _ptr(W), _ptr(L), _ptr(p), _ptr(wbar),
                                                        _ptr(reg), _ptr(drift), C.byref(used),
                                                        int(int(wl.optimistic) == 2))
        if bad:
            raise ValueError("oco_oracle_run_many_optimistic: %d runs failed" % bad)
        return dict(W=W, L=L, p=p, wbar=wbar, regret=reg, max_drift=drift, threads=used.value)
    bad = lib().oco_oracle_run_many(R, d, K, T, float(wl.D), _ptr(eta), float(wl.eps),
                                    LOSS_ID[wl.loss], int(bool(wl.x_shared)),
                                    _ptr(x), _ptr(col), _ptr(val), nnz, _ptr(y), _ptr(u),
                                    _ptr(seg_start), S, int(norm_every), int(threads),
                                    _ptr(W), _ptr(L), _ptr(p), _ptr(wbar), _ptr(reg), _ptr(drift),
                                    C.byref(used))
    if bad:
        raise ValueError("oco_oracle_run_many: %d runs failed" % bad)
    return dict(W=W, L=L, p=p, wbar=wbar, regret=reg, max_drift=drift, threads=used.value)
