"""Host-side checks of the C-ABI boundary that need no GPU: the library loads, exports every
symbol the header declares, sizes workspaces, and rejects bad configurations before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_2605_06113_amd import binding, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "br.h")).read()
    declared = set(re.findall(r"^\s*(?:uint64_t|int32_t|void)\s+(br_[a-z_]+)\s*\(", hdr, re.M))
    assert declared == set(binding.EXPORTS)
    lib = binding.load()
    for name in declared:
        assert hasattr(lib, name)


def test_struct_sizes_match_header():
    assert C.sizeof(binding.Config) == 14 * 4 + 3 * 8 + 2 * 8 + 2 * 4
    assert C.sizeof(binding.Arrivals) == 5 * 8 + 8
    assert C.sizeof(binding.StepOut) == 6 * 8
    assert C.sizeof(binding.Layout) == 15 * 8 + 16


def test_workspace_bytes_scale():
    c4 = binding.workspace_bytes(wl.config("c4"))
    # two int32 slot tables of 4096 x 16 x 144 dominate
    assert 2 * 4096 * 16 * 144 * 4 <= c4 <= 2 * 4096 * 16 * 144 * 4 * 1.3
    assert binding.workspace_bytes(wl.config("c5")) > binding.workspace_bytes(wl.config("c1"))
    assert binding.workspace_bytes(wl.config("c4")) % 256 == 0


@pytest.mark.parametrize("bad", [dict(G=0), dict(G=65), dict(B=0), dict(B=1025), dict(max_wait=0),
                                 dict(max_wait=2049), dict(H=9), dict(H=129, pred_mode=1), dict(H=-1), dict(R_max=0), dict(R_max=33), dict(H=80, pred_mode=1, R_max=17),
                                 dict(n_inst=0), dict(token_watermark=-1), dict(pred_mode=2), dict(H=4, pred_mode=4),
                                 dict(H=2, alpha=0.0), dict(H=2, gamma=0.0), dict(H=2, gamma=1.5)])
def test_invalid_config_rejected(bad):
    cfg = wl.config("c1", **bad)
    assert binding.workspace_bytes(cfg) == 0
    lib = binding.load()
    c = binding.make_config(cfg, workspace=256, workspace_bytes=1 << 30)
    ctx = C.c_void_p()
    assert lib.br_init(C.byref(c), None, C.byref(ctx)) == binding.BR_EINVAL
    assert not ctx.value


def test_long_horizon_config():
    """Horizons up to 128 are accepted with a direct or maintained estimate (a hazard per offset only up to 8);
    the workspace grows by the projection rows and the discount table."""
    short = binding.workspace_bytes(wl.config("c3", H=8, pred_mode=1))
    long_ = binding.workspace_bytes(wl.config("c3", H=80, pred_mode=1))
    assert short > 0 and long_ > short
    assert binding.workspace_bytes(wl.config("c3", H=128, pred_mode=1)) > long_
    assert binding.workspace_bytes(wl.config("c3", H=80, pred_mode=0)) == 0


def test_init_argument_errors():
    lib = binding.load()
    cfg = wl.config("c1")
    need = binding.workspace_bytes(cfg)
    ctx = C.c_void_p()
    c = binding.make_config(cfg, workspace=0, workspace_bytes=need)
    assert lib.br_init(C.byref(c), None, C.byref(ctx)) == binding.BR_EINVAL          # null workspace
    c = binding.make_config(cfg, workspace=4096 + 4, workspace_bytes=need)
    assert lib.br_init(C.byref(c), None, C.byref(ctx)) == binding.BR_EINVAL          # misaligned
    c = binding.make_config(cfg, workspace=4096, workspace_bytes=need - 1)
    assert lib.br_init(C.byref(c), None, C.byref(ctx)) == binding.BR_ENOMEM          # too small
    assert lib.br_route_step(None, None, None) == binding.BR_EINVAL
    assert lib.br_advance_decode(None, 1) == binding.BR_EINVAL
    assert lib.br_route_advance(None, None, None, 1) == binding.BR_EINVAL
    lib.br_free(None)                                                                  # allowed


def test_no_cpu_fallback_when_library_missing(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libbr_hip.so")
    with pytest.raises(RuntimeError):
        binding.load()


def test_binding_checks_sizes_before_anything_reaches_a_kernel():
    """The C ABI takes bare pointers; the Python side refuses arrays whose shapes do not match."""
    import numpy as np
    from paper_2605_06113_amd import workloads as wl
    a = wl.Arrivals(count=np.zeros(2, np.int32), s=np.ones((2, 5), np.int32), o=np.ones((2, 5), np.int32),
                    id=np.zeros((2, 5), np.int32), pred=None)
    binding.DeviceArrivals(a, "cpu", 0)
    with pytest.raises(binding.BrError):
        binding.DeviceArrivals(a, "cpu", 4)                       # predictions missing
    a.pred = np.zeros((2, 5, 3), np.float32)
    with pytest.raises(binding.BrError):
        binding.DeviceArrivals(a, "cpu", 4)                       # wrong width
    a.o = np.ones((2, 4), np.int32)
    with pytest.raises(binding.BrError):
        binding.DeviceArrivals(a, "cpu", 0)
