"""Thin ctypes binding over liboco.so: the same calls as include/oco.h, argument
marshalling only.  PyTorch is used for device memory and streams; every step
of the learner runs in the library's HIP kernels.  There is no fallback: if the
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
# OCO_LIB overrides the library path (to try a differently tuned build of the same sources)
LIB_PATH = os.environ.get("OCO_LIB") or os.path.join(HERE, "liboco.so")

OCO_OK, OCO_EINVAL, OCO_ESEQ, OCO_ERANGE, OCO_ENOMEM, OCO_EHIP, OCO_ENOCOMP, OCO_EUNSUPPORTED = (
    0, -1, -2, -3, -4, -5, -6, -7)
LOSS_ID = {"linear": 0, "squared": 1, "logistic": 2}
# oco_option keys (include/oco.h)
OPT = dict(meta_beside=0, dense_path=1, dense_wpb=2, comparator_gemm=3, dense_half=4, dense_pieces=5,
           sparse_lpw=6, sparse_pipe=7, verbose=8, window_resident=9, sparse_fetch=10)
OCO_STATIC_WS_BYTES = 64 << 20
EXPORTS = ("oco_step_grid", "oco_paper_num_learners", "oco_workspace_bytes", "oco_create",
           "oco_create_static", "oco_set_option",
           "oco_set_comparator", "oco_run_rounds", "oco_regret", "oco_get_state",
           "oco_cum_losses", "oco_accel_bounds", "oco_reset", "oco_set_timing", "oco_last_timing", "oco_last_kernel_timing",
           "oco_rounds_done", "oco_destroy", "oco_strerror",
           "sd_verify", "sd_acceptance", "sd_strerror")


class OcoConfig(C.Structure):
    _fields_ = [("d", C.c_int64), ("K", C.c_int64), ("T", C.c_int64), ("R", C.c_int64),
                ("D", C.c_double), ("G", C.c_double), ("eta", C.POINTER(C.c_double)),
                ("eps", C.c_double), ("loss", C.c_int32), ("x_shared", C.c_int32),
                ("sparse_nnz", C.c_int32), ("optimistic", C.c_int32), ("n_max", C.c_int64)]


class OcoRounds(C.Structure):
    _fields_ = [("x", C.c_void_p), ("col", C.c_void_p), ("val", C.c_void_p), ("y", C.c_void_p),
                ("x_run_stride", C.c_int64), ("y_run_stride", C.c_int64)]


class OcoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, strerror(status), status))


_lib = None


def lib() -> C.CDLL:
    """Load liboco.so (built by paper_2603_12617_amd/build.py); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("liboco.so is not built: run `python -m paper_2603_12617_amd.build` "
                              "(or __graft_entry__.build()) first; there is no CPU fallback")
        # PyTorch ships its own HIP runtime.  It must be in the process before liboco.so is
        # loaded so that both resolve to the SAME runtime: device pointers and streams that
        # torch hands us are only meaningful to the runtime that created them.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, i64, dbl = C.c_void_p, C.c_int64, C.c_double
        L.oco_step_grid.restype = C.c_int
        L.oco_step_grid.argtypes = [dbl, dbl, i64, i64, vp]
        L.oco_paper_num_learners.restype = i64
        L.oco_paper_num_learners.argtypes = [i64]
        L.oco_workspace_bytes.restype = C.c_size_t
        L.oco_workspace_bytes.argtypes = [C.POINTER(OcoConfig)]
        L.oco_create.restype = C.c_int
        L.oco_create.argtypes = [C.POINTER(OcoConfig), vp, C.c_size_t, vp, C.POINTER(vp)]
        L.oco_create_static.restype = C.c_int
        L.oco_create_static.argtypes = [C.POINTER(OcoConfig), vp, C.POINTER(vp)]
        L.oco_set_option.restype = C.c_int
        L.oco_set_option.argtypes = [vp, C.c_int, i64]
        L.oco_set_comparator.restype = C.c_int
        L.oco_set_comparator.argtypes = [vp, vp, vp, i64]
        L.oco_run_rounds.restype = C.c_int
        L.oco_run_rounds.argtypes = [vp, C.POINTER(OcoRounds), i64, i64]
        L.oco_regret.restype = C.c_int
        L.oco_regret.argtypes = [vp, vp]
        L.oco_cum_losses.restype = C.c_int
        L.oco_cum_losses.argtypes = [vp, vp]
        L.oco_accel_bounds.restype = C.c_int
        L.oco_accel_bounds.argtypes = [vp, i64, C.c_double, vp]
        L.oco_get_state.restype = C.c_int
        L.oco_get_state.argtypes = [vp, vp, vp, vp]
        L.oco_reset.restype = C.c_int
        L.oco_reset.argtypes = [vp]
        L.oco_set_timing.restype = C.c_int
        L.oco_set_timing.argtypes = [vp, C.c_int]
        L.oco_last_timing.restype = C.c_int
        L.oco_last_timing.argtypes = [vp, vp]
        L.oco_last_kernel_timing.restype = C.c_int
        L.oco_last_kernel_timing.argtypes = [vp, vp, vp, vp, vp]
        L.sd_verify.restype = C.c_int
        L.sd_verify.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, vp, vp, vp]
        L.sd_acceptance.restype = C.c_int
        L.sd_acceptance.argtypes = [vp, vp, i64, i64, i64, vp, vp]
        L.sd_strerror.restype = C.c_char_p
        L.sd_strerror.argtypes = [C.c_int]
        L.oco_rounds_done.restype = i64
        L.oco_rounds_done.argtypes = [vp]
        L.oco_destroy.restype = None
        L.oco_destroy.argtypes = [vp]
        L.oco_strerror.restype = C.c_char_p
        L.oco_strerror.argtypes = [C.c_int]
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().oco_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != OCO_OK:
        raise OcoError(status, where)


def make_config(*, d, K, T, R, D, G, eta: Sequence[float], eps, loss, x_shared=True, nnz=0,
                n_max=0, optimistic=False):
    """Returns (OcoConfig, keepalive) -- keepalive owns the eta array."""
    eta_arr = (C.c_double * len(eta))(*[float(e) for e in eta])
    cfg = OcoConfig(int(d), int(K), int(T), int(R), float(D), float(G),
                    C.cast(eta_arr, C.POINTER(C.c_double)), float(eps),
                    LOSS_ID[loss] if isinstance(loss, str) else int(loss), int(bool(x_shared)),
                    int(nnz), int(optimistic), int(n_max))
    return cfg, eta_arr


def oco_step_grid(D: float, G: float, T: int, K: int) -> np.ndarray:
    out = np.empty(max(K, 0), dtype=np.float64)
    _check(lib().oco_step_grid(float(D), float(G), int(T), int(K), out.ctypes.data), "oco_step_grid")
    return out


def oco_paper_num_learners(T: int) -> int:
    return int(lib().oco_paper_num_learners(int(T)))


def oco_workspace_bytes(cfg: OcoConfig) -> int:
    return int(lib().oco_workspace_bytes(C.byref(cfg)))


def _dptr(t) -> Optional[int]:
    """Device (or None) pointer of a torch tensor."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous()
    return t.data_ptr()


def oco_create(cfg: OcoConfig, ws, stream=None) -> int:
    """ws: torch uint8 CUDA tensor of >= oco_workspace_bytes(cfg) bytes.  Returns the handle."""
    h = C.c_void_p()
    sp = None if stream is None else stream.cuda_stream
    _check(lib().oco_create(C.byref(cfg), _dptr(ws), ws.numel() * ws.element_size(), sp, C.byref(h)),
           "oco_create")
    return h.value


def oco_create_static(cfg: OcoConfig, stream=None) -> int:
    """The same state in the library's own device array (no workspace from the caller)."""
    h = C.c_void_p()
    sp = None if stream is None else stream.cuda_stream
    _check(lib().oco_create_static(C.byref(cfg), sp, C.byref(h)), "oco_create_static")
    return h.value


def oco_set_option(h: int, key, value: int) -> None:
    """key: an oco_option number or its name in OPT."""
    k = OPT[key] if isinstance(key, str) else int(key)
    _check(lib().oco_set_option(h, k, int(value)), "oco_set_option")


def oco_set_comparator(h: int, u, seg_start) -> None:
    seg = np.ascontiguousarray(seg_start, dtype=np.int64)
    _check(lib().oco_set_comparator(h, _dptr(u), seg.ctypes.data, seg.size), "oco_set_comparator")


def oco_run_rounds(h: int, t0: int, n: int, *, x=None, col=None, val=None, y=None,
                   x_ptr=None, col_ptr=None, val_ptr=None, y_ptr=None,
                   x_run_stride=0, y_run_stride=0) -> None:
    """Tensors (whole slices) or raw device addresses (for slices of resident arrays)."""
    rd = OcoRounds(x_ptr if x_ptr is not None else _dptr(x),
                   col_ptr if col_ptr is not None else _dptr(col),
                   val_ptr if val_ptr is not None else _dptr(val),
                   y_ptr if y_ptr is not None else _dptr(y),
                   int(x_run_stride), int(y_run_stride))
    _check(lib().oco_run_rounds(h, C.byref(rd), int(t0), int(n)), "oco_run_rounds")


def oco_regret(h: int, R: int) -> np.ndarray:
    out = np.empty(R, dtype=np.float64)
    _check(lib().oco_regret(h, out.ctypes.data), "oco_regret")
    return out


def oco_cum_losses(h: int, R: int, K: int) -> np.ndarray:
    out = np.empty((R, K), dtype=np.float64)
    _check(lib().oco_cum_losses(h, out.ctypes.data), "oco_cum_losses")
    return out


def oco_accel_bounds(h: int, k: int, alpha: float, out) -> None:
    """out: device float64 tensor [R][4] (length bounds, rate bounds of Lemma 1 / Theorem 1)."""
    _check(lib().oco_accel_bounds(h, int(k), float(alpha), _dptr(out)), "oco_accel_bounds")


def oco_get_state(h: int, W=None, p=None, wbar=None) -> None:
    _check(lib().oco_get_state(h, _dptr(W), _dptr(p), _dptr(wbar)), "oco_get_state")


def oco_reset(h: int) -> None:
    _check(lib().oco_reset(h), "oco_reset")


def oco_set_timing(h: int, enable: bool) -> None:
    _check(lib().oco_set_timing(h, int(bool(enable))), "oco_set_timing")


def oco_last_timing(h: int) -> np.ndarray:
    """[ms of the round kernel, ms of the meta kernel] of the last oco_run_rounds call."""
    out = np.zeros(2, dtype=np.float32)
    _check(lib().oco_last_timing(h, out.ctypes.data), "oco_last_timing")
    return out


def oco_last_kernel_timing(h: int) -> dict:
    """The dominant kernel of the last timed call alone: its name, the launches of it in the call,
    how many of them were timed and their summed duration in ms."""
    ms, timed, launches, name = C.c_float(0), C.c_int(0), C.c_int(0), C.c_char_p()
    _check(lib().oco_last_kernel_timing(h, C.addressof(ms), C.addressof(timed), C.addressof(launches), C.addressof(name)),
           "oco_last_kernel_timing")
    return dict(kernel=(name.value or b"").decode(), ms_sum=float(ms.value), timed=int(timed.value), launches=int(launches.value))


def oco_rounds_done(h: int) -> int:
    return int(lib().oco_rounds_done(h))


def oco_destroy(h: Optional[int]) -> None:
    if h:
        lib().oco_destroy(h)


class Simulation:
    """Holds one workload resident on the GPU and drives it through the C ABI.

    `wl` is a workloads.Workload, `data` the dict from workloads.generate (numpy).  All
    arithmetic happens inside oco_run_rounds / oco_get_state; this class only uploads the
    arrays, slices them by pointer arithmetic and downloads results."""

    def __init__(self, wl, data, n_max: int = 0, device: str = "cuda:0", stream=None, options=None,
                 static: bool = False):
        import torch
        self.torch = torch
        self.wl = wl
        self.dev = torch.device(device)
        self.stream = stream
        up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)
        self.x, self.col, self.val, self.y, self.u = (up(data.get(k)) for k in ("x", "col", "val", "y", "u"))
        self.seg_start = np.ascontiguousarray(data["seg_start"], dtype=np.int64)
        self.cfg, self._keep = make_config(d=wl.d, K=wl.K, T=wl.T, R=wl.R, D=wl.D, G=wl.G, eta=wl.eta,
                                           eps=wl.eps, loss=wl.loss, x_shared=wl.x_shared, nnz=wl.nnz,
                                           n_max=n_max, optimistic=int(getattr(wl, "optimistic", 0)))
        nbytes = oco_workspace_bytes(self.cfg)
        if nbytes == 0:
            raise OcoError(OCO_EINVAL, "oco_workspace_bytes")
        if static:
            self.ws = None
            self.h = oco_create_static(self.cfg, stream)
        else:
            self.ws = torch.empty(nbytes, dtype=torch.uint8, device=self.dev)
            self.h = oco_create(self.cfg, self.ws, stream)
        for k, v in (options or {}).items():
            oco_set_option(self.h, k, v)
        oco_set_comparator(self.h, self.u, self.seg_start)

    def run(self, t0: int, n: int) -> None:
        wl = self.wl
        kw = {}
        if wl.nnz:
            kw["col_ptr"] = self.col.data_ptr() + 4 * t0 * wl.nnz
            kw["val_ptr"] = self.val.data_ptr() + 4 * t0 * wl.nnz
        else:
            kw["x_ptr"] = self.x.data_ptr() + 4 * t0 * wl.d
            kw["x_run_stride"] = 0 if wl.x_shared else wl.T * wl.d
        if self.y is not None:
            kw["y_ptr"] = self.y.data_ptr() + 4 * t0
            kw["y_run_stride"] = wl.T
        oco_run_rounds(self.h, t0, n, **kw)

    def run_all(self, chunk: int = 0) -> None:
        T = self.wl.T
        chunk = chunk or T
        t = oco_rounds_done(self.h)
        while t < T:
            n = min(chunk, T - t)
            self.run(t, n)
            t += n

    def regret(self) -> np.ndarray:
        return oco_regret(self.h, self.wl.R)

    def cum_losses(self) -> np.ndarray:
        return oco_cum_losses(self.h, self.wl.R, self.wl.K)

    def accel_bounds(self, k: int, alpha: float) -> np.ndarray:
        out = self.torch.empty((self.wl.R, 4), dtype=self.torch.float64, device=self.dev)
        oco_accel_bounds(self.h, k, alpha, out)
        self.sync()
        return out.cpu().numpy()

    def state(self, want_W: bool = True):
        torch, wl = self.torch, self.wl
        W = torch.empty((wl.R, wl.K, wl.d), dtype=torch.float32, device=self.dev) if want_W else None
        p = torch.empty((wl.R, wl.K), dtype=torch.float32, device=self.dev)
        wbar = torch.empty((wl.R, wl.d), dtype=torch.float32, device=self.dev)
        oco_get_state(self.h, W, p, wbar)
        self.sync()
        return W, p, wbar

    def reset(self) -> None:
        oco_reset(self.h)

    def sync(self) -> None:
        if self.stream is None:
            self.torch.cuda.synchronize(self.dev)
        else:
            self.stream.synchronize()

    def close(self) -> None:
        if getattr(self, "h", None):
            self.sync()
            oco_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---------------------------------------------------------------------------
# Verification step of speculative decoding (include/specdec.h)
class SdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, lib().sd_strerror(status).decode(), status))


def _stream_ptr(stream):
    return None if stream is None else stream.cuda_stream


def sd_verify(p, q, tok, r, u, n_out, next_out, stream=None) -> None:
    """p [B][k+1][V] f32, q [B][k][V] f32, tok [B][k] i32, r [B][k] f32, u [B] u32 (as int32/uint32
    torch tensor), n_out / next_out [B] i32 -- all CUDA tensors.  Asynchronous."""
    B, k, V = q.shape
    assert tuple(p.shape) == (B, k + 1, V) and tuple(tok.shape) == (B, k) and tuple(r.shape) == (B, k)
    rc = lib().sd_verify(_dptr(p), _dptr(q), _dptr(tok), _dptr(r), _dptr(u), B, k, V,
                         _dptr(n_out), _dptr(next_out), _stream_ptr(stream))
    if rc != 0:
        raise SdError(rc, "sd_verify")


def sd_acceptance(p, q, acc_out, stream=None) -> None:
    """acc_out [B][k] f64 = sum_x min(p, q) per draft position.  Asynchronous."""
    B, k, V = q.shape
    rc = lib().sd_acceptance(_dptr(p), _dptr(q), B, k, V, _dptr(acc_out), _stream_ptr(stream))
    if rc != 0:
        raise SdError(rc, "sd_acceptance")
