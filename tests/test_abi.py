"""The C-ABI boundary without a GPU: the library loads, exports every function the header
declares, and rejects bad arguments on the host before any device work."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

from paper_2603_12617_amd import binding as B
from paper_2603_12617_amd import workloads as WL

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for header, prefix in (("oco.h", "oco"), ("specdec.h", "sd")):
        src = open(os.path.join(ROOT, "include", header)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names |= set(re.findall(r"\b(%s_[a-z_]+)\s*\(" % prefix, src))
    return sorted(names)


def test_library_exports_every_declared_function():
    names = _declared()
    assert len(names) >= 12
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(B.EXPORTS)


def test_status_strings():
    seen = {B.strerror(s) for s in range(0, -8, -1)}
    assert len(seen) == 8 and "unknown status" not in seen
    assert B.strerror(-99) == "unknown status"


def test_step_grid_and_learner_count():
    np.testing.assert_allclose(B.oco_step_grid(1.0, 1.0, 10000, 15), WL.step_grid(1.0, 1.0, 10000, 15), rtol=1e-15)
    np.testing.assert_allclose(B.oco_step_grid(2.0, 4.0, 100, 3), [0.05, 0.1, 0.2], rtol=1e-15)
    assert [B.oco_paper_num_learners(T) for T in (1000, 10 ** 4, 10 ** 5)] == [6, 8, 10]
    with pytest.raises(B.OcoError):
        B.oco_step_grid(0.0, 1.0, 10, 2)
    with pytest.raises(B.OcoError):
        B.oco_step_grid(1.0, 1.0, 0, 2)


def _cfg(**over):
    base = dict(d=100, K=3, T=1000, R=4, D=1.0, G=1.0, eta=[0.01, 0.02, 0.04], eps=0.1, loss="squared")
    base.update(over)
    return B.make_config(**base)


def test_workspace_bytes_is_zero_for_bad_configs():
    ok, keep = _cfg()
    assert B.oco_workspace_bytes(ok) > 4 * 4 * 3 * 100
    for bad in (dict(d=0), dict(K=0), dict(T=0), dict(R=0), dict(D=0.0), dict(D=float("nan")),
                dict(D=float("inf")), dict(G=-1.0), dict(eps=-0.1), dict(eps=float("nan")),
                dict(loss=7), dict(eta=[0.1, -0.2, 0.3]), dict(eta=[0.1, float("inf"), 0.3]),
                dict(n_max=-1), dict(d=4097), dict(d=4100, x_shared=False), dict(d=8192, x_shared=False, optimistic=True),
                dict(d=65540), dict(K=65, eta=[0.1] * 65),
                dict(nnz=65, d=1 << 20), dict(nnz=8, d=4), dict(nnz=8, d=1 << 20, x_shared=False)):
        cfg, keep = _cfg(**bad)
        assert B.oco_workspace_bytes(cfg) == 0, bad
    cfg, keep = _cfg()
    for bad_opt in (3, -1):
        cfg.optimistic = bad_opt
        assert B.oco_workspace_bytes(cfg) == 0
    # optimism at both levels keeps the last observed losses beside the cumulative ones
    cfg.optimistic = 1
    one_level = B.oco_workspace_bytes(cfg)
    cfg.optimistic = 2
    assert B.oco_workspace_bytes(cfg) > one_level > 0
    # a shared stream may be wider than one wavefront's registers (iterates streamed from HBM)
    for good in (dict(d=4096, x_shared=False), dict(d=8192), dict(d=65536), dict(d=8192, optimistic=True)):
        cfg, keep = _cfg(**good)
        assert B.oco_workspace_bytes(cfg) > 0, good
    cfg, keep = _cfg(d=1 << 20, nnz=8)
    plain_sparse = B.oco_workspace_bytes(cfg)
    cfg.optimistic = 1
    assert B.oco_workspace_bytes(cfg) > plain_sparse > 0
    plain, k1 = _cfg()
    opt, k2 = _cfg()
    opt.optimistic = 1
    assert B.oco_workspace_bytes(opt) > B.oco_workspace_bytes(plain)
    assert B.lib().oco_workspace_bytes(None) == 0


def test_workspace_grows_with_the_call_size_and_covers_the_state():
    small, k1 = _cfg(n_max=64)
    big, k2 = _cfg(n_max=0)
    assert B.oco_workspace_bytes(small) < B.oco_workspace_bytes(big)
    c5, k3 = _cfg(d=1 << 20, K=8, R=16, T=100000, eta=[0.1] * 8, nnz=32, n_max=1000)
    assert B.oco_workspace_bytes(c5) >= 4 * (1 << 20) * 128          # the 512 MB iterate block


def test_create_rejects_bad_arguments_on_the_host():
    L = B.lib()
    cfg, keep = _cfg()
    need = B.oco_workspace_bytes(cfg)
    h = C.c_void_p()
    assert L.oco_create(C.byref(cfg), 256, need, None, None) == B.OCO_EINVAL
    assert L.oco_create(None, 256, need, None, C.byref(h)) == B.OCO_EINVAL
    assert L.oco_create(C.byref(cfg), None, need, None, C.byref(h)) == B.OCO_EINVAL
    assert L.oco_create(C.byref(cfg), 264, need, None, C.byref(h)) == B.OCO_EINVAL      # misaligned
    assert L.oco_create(C.byref(cfg), 256, need - 1, None, C.byref(h)) == B.OCO_ENOMEM
    bad, keep2 = _cfg(d=4097)
    assert L.oco_create(C.byref(bad), 256, 1 << 40, None, C.byref(h)) == B.OCO_EUNSUPPORTED
    assert h.value is None
    # NULL handles are rejected, not dereferenced
    assert L.oco_run_rounds(None, None, 0, 0) == B.OCO_EINVAL
    assert L.oco_regret(None, None) == B.OCO_EINVAL
    assert L.oco_get_state(None, None, None, None) == B.OCO_EINVAL
    assert L.oco_set_comparator(None, None, None, 1) == B.OCO_EINVAL
    assert L.oco_reset(None) == B.OCO_EINVAL
    assert L.oco_set_timing(None, 1) == B.OCO_EINVAL
    assert L.oco_last_timing(None, None) == B.OCO_EINVAL
    assert L.oco_last_kernel_timing(None, None, None, None, None) == B.OCO_EINVAL
    assert L.oco_rounds_done(None) == B.OCO_EINVAL
    assert L.oco_set_option(None, 0, 0) == B.OCO_EINVAL
    L.oco_destroy(None)


def test_static_create_rejects_bad_arguments_and_oversize_configs_on_the_host():
    L = B.lib()
    h = C.c_void_p()
    cfg, keep = _cfg()
    assert L.oco_create_static(C.byref(cfg), None, None) == B.OCO_EINVAL
    assert L.oco_create_static(None, None, C.byref(h)) == B.OCO_EINVAL
    bad, keep2 = _cfg(d=4097)
    assert L.oco_create_static(C.byref(bad), None, C.byref(h)) == B.OCO_EUNSUPPORTED
    # a state larger than the library's own device array: refused before any device call
    big, keep3 = _cfg(d=4096, K=16, R=1024, eta=[0.1] * 16)
    assert B.oco_workspace_bytes(big) > B.OCO_STATIC_WS_BYTES
    assert L.oco_create_static(C.byref(big), None, C.byref(h)) == B.OCO_ENOMEM
    # ... and one whose state fits but whose call size does not, until n_max is lowered
    mid, keep4 = _cfg(d=100, K=15, R=64, T=100000, eta=[0.1] * 15, x_shared=False)
    assert L.oco_create_static(C.byref(mid), None, C.byref(h)) == B.OCO_ENOMEM
    mid.n_max = 4096
    assert 0 < B.oco_workspace_bytes(mid) <= B.OCO_STATIC_WS_BYTES
    assert h.value is None


def test_specdec_host_validation():
    L = B.lib()
    one = C.c_void_p(256)          # any non-null, aligned address: rejected before it is touched
    assert L.sd_verify(None, one, one, one, one, 1, 1, 8, one, one, None) == -1
    assert L.sd_verify(one, one, one, one, one, 0, 1, 8, one, one, None) == -1
    assert L.sd_verify(one, one, one, one, one, 1, 65, 8, one, one, None) == -2
    assert L.sd_verify(one, one, one, one, one, 1, 4, 262145, one, one, None) == -2
    assert L.sd_verify(C.c_void_p(258), one, one, one, one, 1, 4, 8, one, one, None) == -1
    assert L.sd_acceptance(one, None, 1, 1, 8, one, None) == -1
    assert L.sd_acceptance(one, one, 1, 1, 8, C.c_void_p(260), None) == -1
    assert L.sd_acceptance(one, one, 1, 0, 8, one, None) == -1
    assert L.sd_strerror(0) == b"ok" and L.sd_strerror(-7) == b"unknown status"
