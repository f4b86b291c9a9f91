"""Thin ctypes binding over the C-ABI HIP library (include/br.h).

Argument marshalling only: every step of the path runs in the library's kernels.
PyTorch is used for device memory and the stream handle, nothing else.  There is
no CPU fallback: if the library is missing or a symbol is not exported, loading
fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbr_hip.so")

NSTATS = 16
NKERNELS = 7
KERNEL_NAMES = ("project", "score", "assign", "advance", "init", "bypass", "baseline")
POLICY = dict(random=0, rr=1, p2c=2, jsq=3)
ST = dict(admitted=0, deferred=1, dropped=2, stage1=3, stage2_pops=4, guard=5, overcap=6,
          I_before=7, I_after=8, spread=9, qlen=10, workers_dropped=11, load_range=12)
BR_OK, BR_EINVAL, BR_ENOMEM, BR_EHIP, BR_ELIMIT = 0, -1, -2, -3, -4

EXPORTS = ("br_workspace_bytes", "br_init", "br_route_step", "br_route_step_static", "br_route_advance", "br_route_bypass", "br_route_baseline", "br_advance_decode", "br_free",
           "br_last_hip_error", "br_get_layout", "br_profile_enable", "br_profile_read")

_P = C.c_void_p


class Config(C.Structure):
    _fields_ = [("n_inst", C.c_int32), ("G", C.c_int32), ("B", C.c_int32), ("max_wait", C.c_int32),
                ("H", C.c_int32), ("S_greedy", C.c_int32), ("R_max", C.c_int32),
                ("token_watermark", C.c_int32), ("token_cap", C.c_int32), ("pred_mode", C.c_int32),
                ("alpha", C.c_float), ("beta", C.c_float), ("gamma", C.c_float), ("gate_pfin", C.c_float),
                ("stream", _P), ("workspace", _P), ("workspace_bytes", C.c_uint64),
                ("hist", _P), ("hist_sum", _P), ("hist_n", C.c_int32), ("refresh_period", C.c_int32)]


class InitState(C.Structure):
    _fields_ = [("n", _P), ("kv", _P), ("rem", _P), ("pred", _P)]


class Arrivals(C.Structure):
    _fields_ = [("count", _P), ("s", _P), ("o", _P), ("id", _P), ("pred", _P),
                ("arr_cap", C.c_int32), ("pad", C.c_int32)]


class StepOut(C.Structure):
    _fields_ = [("assign", _P), ("assign_id", _P), ("stats", _P), ("F", _P), ("best_g", _P), ("best_i", _P)]


class Layout(C.Structure):
    _fields_ = [(k, C.c_uint64) for k in ("L", "n", "kv", "rem", "pred", "qlen", "qs", "qo", "qid", "qpred",
                                          "Lh", "Mh", "mh", "minm", "total_bytes")] + \
               [("B_stride", C.c_int32), ("P", C.c_int32), ("Pq", C.c_int32), ("pad", C.c_int32)]


_lib = None


def load():
    """Load the library and bind every symbol include/br.h declares (raises if one is missing)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not built: run `python __graft_entry__.py` (hipcc, gfx950) first")
    lib = C.CDLL(LIB_PATH)
    for name in EXPORTS:
        getattr(lib, name)  # AttributeError if not exported
    lib.br_workspace_bytes.restype = C.c_uint64
    lib.br_workspace_bytes.argtypes = [C.POINTER(Config)]
    lib.br_init.restype = C.c_int32
    lib.br_init.argtypes = [C.POINTER(Config), C.POINTER(InitState), C.POINTER(_P)]
    lib.br_route_step.restype = C.c_int32
    lib.br_route_step.argtypes = [_P, C.POINTER(Arrivals), C.POINTER(StepOut)]
    lib.br_route_step_static.restype = C.c_int32
    lib.br_route_step_static.argtypes = [_P, C.POINTER(Arrivals), C.POINTER(StepOut)]
    lib.br_route_advance.restype = C.c_int32
    lib.br_route_advance.argtypes = [_P, C.POINTER(Arrivals), C.POINTER(StepOut), C.c_int32]
    lib.br_route_bypass.restype = C.c_int32
    lib.br_route_bypass.argtypes = [_P, C.POINTER(Arrivals), C.POINTER(StepOut)]
    lib.br_route_baseline.restype = C.c_int32
    lib.br_route_baseline.argtypes = [_P, C.POINTER(Arrivals), C.POINTER(StepOut), C.c_int32, C.c_uint64]
    lib.br_advance_decode.restype = C.c_int32
    lib.br_advance_decode.argtypes = [_P, C.c_int32]
    lib.br_free.restype = None
    lib.br_free.argtypes = [_P]
    lib.br_last_hip_error.restype = C.c_int32
    lib.br_last_hip_error.argtypes = [_P]
    lib.br_get_layout.restype = C.c_int32
    lib.br_get_layout.argtypes = [_P, C.POINTER(Layout)]
    lib.br_profile_enable.restype = C.c_int32
    lib.br_profile_enable.argtypes = [_P, C.c_int32]
    lib.br_profile_read.restype = C.c_int32
    lib.br_profile_read.argtypes = [_P, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    _lib = lib
    return lib


def make_config(cfg, stream=0, workspace=0, workspace_bytes=0, hist=0, hist_sum=0, hist_n=0) -> Config:
    """cfg: any object with the workloads.RouteConfig fields; hist*: device pointers (pred_mode 2)."""
    return Config(hist=hist, hist_sum=hist_sum, hist_n=hist_n, refresh_period=int(getattr(cfg, "refresh_eff", 1)),
                  n_inst=cfg.n_inst, G=cfg.G, B=cfg.B, max_wait=cfg.max_wait, H=cfg.H,
                  S_greedy=cfg.s_greedy, R_max=cfg.R_max, token_watermark=cfg.token_watermark,
                  token_cap=cfg.token_cap, pred_mode=cfg.pred_mode, alpha=cfg.alpha, beta=cfg.beta_eff,
                  gamma=cfg.gamma, gate_pfin=cfg.gate_pfin, stream=stream, workspace=workspace,
                  workspace_bytes=workspace_bytes)


def workspace_bytes(cfg, hist_n: int = 0) -> int:
    # the size does not depend on the history's contents; any non-null address passes validation
    c = make_config(cfg, hist=256 if hist_n else 0, hist_sum=256 if hist_n else 0, hist_n=hist_n)
    return int(load().br_workspace_bytes(C.byref(c)))


class BrError(RuntimeError):
    pass


def _check(rc: int, what: str, ctx=None):
    if rc != BR_OK:
        hip = load().br_last_hip_error(ctx) if ctx else 0
        raise BrError(f"{what} failed: rc={rc} hip_error={hip}")


class DeviceArrivals:
    """One batch of arrivals resident on the device."""

    def __init__(self, arr, device, P: int):
        import torch
        # the C ABI takes bare pointers: sizes are checked here, before anything reaches a kernel
        n_inst, cap = np.shape(arr.s)
        for name in ("o", "id"):
            if np.shape(getattr(arr, name)) != (n_inst, cap):
                raise BrError(f"arrivals.{name} must have shape {(n_inst, cap)}")
        if np.shape(arr.count) != (n_inst,):
            raise BrError(f"arrivals.count must have shape {(n_inst,)}")
        if P and (arr.pred is None or np.shape(arr.pred) != (n_inst, cap, P)):
            raise BrError(f"arrivals.pred must have shape {(n_inst, cap, P)}")
        self.count = torch.as_tensor(np.ascontiguousarray(arr.count, np.int32), device=device)
        self.s = torch.as_tensor(np.ascontiguousarray(arr.s, np.int32), device=device)
        self.o = torch.as_tensor(np.ascontiguousarray(arr.o, np.int32), device=device)
        self.id = torch.as_tensor(np.ascontiguousarray(arr.id, np.int32), device=device)
        self.pred = torch.as_tensor(np.ascontiguousarray(arr.pred, np.float32), device=device) if P else None
        self.arr_cap = int(arr.s.shape[-1])

    def struct(self) -> Arrivals:
        return Arrivals(count=self.count.data_ptr(), s=self.s.data_ptr(), o=self.o.data_ptr(),
                        id=self.id.data_ptr(), pred=self.pred.data_ptr() if self.pred is not None else None,
                        arr_cap=self.arr_cap, pad=0)


class Router:
    """Owns a workspace tensor and a br_ctx; all methods only marshal arguments."""

    def __init__(self, cfg, init=None, device="cuda:0", stream=None, hist=None):
        import torch
        self.torch = torch
        self.lib = load()
        self.cfg = cfg
        self.device = torch.device(device)
        self.N, self.G, self.B, self.Q, self.H = cfg.n_inst, cfg.G, cfg.B, cfg.max_wait, cfg.H
        self.P = 0 if cfg.H == 0 else {1: 1, 2: 3, 3: 2}.get(cfg.pred_mode, cfg.H)
        self.Pq = 0 if cfg.pred_mode == 2 else self.P
        self._hist = None
        hargs = {}
        if hist is not None:   # sorted output-length history and its prefix sums, resident on the device
            h = np.ascontiguousarray(hist, np.int32)
            hs = np.concatenate([[0], np.cumsum(h, dtype=np.int64)]).astype(np.int64)
            self._hist = (torch.as_tensor(h, device=self.device), torch.as_tensor(hs, device=self.device))
            hargs = dict(hist=self._hist[0].data_ptr(), hist_sum=self._hist[1].data_ptr(), hist_n=len(h))
        nbytes = workspace_bytes(cfg, hist_n=len(hist) if hist is not None else 0)
        if nbytes == 0:
            raise BrError("invalid configuration")
        self.ws = torch.empty(nbytes // 4 + 64, dtype=torch.int32, device=self.device)
        assert self.ws.data_ptr() % 256 == 0
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        c = make_config(cfg, stream=self.stream.cuda_stream, workspace=self.ws.data_ptr(),
                        workspace_bytes=self.ws.numel() * 4, **hargs)
        ini = None
        self._keep = []
        if init is not None:
            if np.shape(init.n) != (self.N, self.G):
                raise BrError(f"init.n must have shape {(self.N, self.G)}")
            for name in ("kv", "rem"):
                if np.shape(getattr(init, name)) != (self.N, self.G, self.B):
                    raise BrError(f"init.{name} must have shape {(self.N, self.G, self.B)}")
            if self.P and (init.pred is None or np.shape(init.pred) != (self.N, self.G, self.B, self.P)):
                raise BrError(f"init.pred must have shape {(self.N, self.G, self.B, self.P)}")
            t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a, dt), device=self.device)
            n, kv, rem = t(init.n, np.int32), t(init.kv, np.int32), t(init.rem, np.int32)
            pred = t(init.pred, np.float32) if self.P else None
            self._keep = [n, kv, rem, pred]
            ini = InitState(n=n.data_ptr(), kv=kv.data_ptr(), rem=rem.data_ptr(),
                            pred=pred.data_ptr() if pred is not None else None)
        ctx = _P()
        _check(self.lib.br_init(C.byref(c), C.byref(ini) if ini is not None else None, C.byref(ctx)), "br_init")
        self.ctx = ctx
        lay = Layout()
        _check(self.lib.br_get_layout(self.ctx, C.byref(lay)), "br_get_layout", self.ctx)
        self.layout = lay
        self.Bs = lay.B_stride
        self._out: Dict[str, object] = {}

    # -- outputs -------------------------------------------------------
    def alloc_outputs(self, scores: bool = True, matrix: bool = True) -> Dict[str, object]:
        torch = self.torch
        N, G, Q = self.N, self.G, self.Q
        out = dict(assign=torch.empty((N, Q), dtype=torch.int32, device=self.device),
                   assign_id=torch.empty((N, Q), dtype=torch.int32, device=self.device),
                   stats=torch.empty((N, NSTATS), dtype=torch.int64, device=self.device))
        if scores:
            out["best_g"] = torch.empty((N, Q), dtype=torch.int32, device=self.device)
            out["best_i"] = torch.empty((N, G), dtype=torch.int32, device=self.device)
            if matrix:
                out["F"] = torch.zeros((N, Q, G), dtype=torch.float32 if self.H > 0 else torch.int32,
                                       device=self.device)
        return out

    @staticmethod
    def out_struct(out) -> StepOut:
        g = lambda k: out[k].data_ptr() if out.get(k) is not None else None
        return StepOut(assign=g("assign"), assign_id=g("assign_id"), stats=g("stats"), F=g("F"),
                       best_g=g("best_g"), best_i=g("best_i"))

    # -- calls ---------------------------------------------------------
    def route_step_device(self, darr: Optional[DeviceArrivals], out) -> None:
        """Enqueue one round; inputs and outputs are device tensors; no synchronisation."""
        a = darr.struct() if darr is not None else None
        o = self.out_struct(out)
        _check(self.lib.br_route_step(self.ctx, C.byref(a) if a is not None else None, C.byref(o)),
               "br_route_step", self.ctx)

    def route_step_static_device(self, darr: Optional[DeviceArrivals], out) -> int:
        """Enqueue one round through the entry point that uses the library's fixed scratch array; returns the
        status code (BR_ELIMIT for contexts it does not serve) instead of raising."""
        a = darr.struct() if darr is not None else None
        o = self.out_struct(out)
        return int(self.lib.br_route_step_static(self.ctx, C.byref(a) if a is not None else None, C.byref(o)))

    def route_advance_device(self, darr: Optional[DeviceArrivals], out, n_steps: int = 1) -> None:
        """Enqueue one round and n_steps decode steps as one launch; no synchronisation."""
        a = darr.struct() if darr is not None else None
        o = self.out_struct(out)
        _check(self.lib.br_route_advance(self.ctx, C.byref(a) if a is not None else None, C.byref(o), int(n_steps)),
               "br_route_advance", self.ctx)

    def route_step(self, arr=None, scores: bool = True, matrix: bool = True, advance: int = 0):
        """Convenience for tests: host arrays in, numpy out (synchronises).  advance > 0 takes the
        fused entry point (round + that many decode steps)."""
        darr = DeviceArrivals(arr, self.device, self.Pq) if arr is not None else None
        out = self.alloc_outputs(scores, matrix)
        if advance > 0:
            self.route_advance_device(darr, out, advance)
        else:
            self.route_step_device(darr, out)
        self.stream.synchronize()
        return {k: v.cpu().numpy() for k, v in out.items()}

    def route_bypass_device(self, darr: DeviceArrivals, out) -> None:
        """Enqueue the pool-bypass dispatch of one batch of arrivals (BR-0); no synchronisation."""
        a = darr.struct()
        o = self.out_struct(out)
        _check(self.lib.br_route_bypass(self.ctx, C.byref(a), C.byref(o)), "br_route_bypass", self.ctx)

    def route_bypass(self, arr):
        """Convenience for tests: host arrays in, numpy out (synchronises)."""
        torch = self.torch
        darr = DeviceArrivals(arr, self.device, 0)
        out = dict(assign=torch.full((self.N, darr.arr_cap), -3, dtype=torch.int32, device=self.device),
                   stats=torch.zeros((self.N, NSTATS), dtype=torch.int64, device=self.device))
        self.route_bypass_device(darr, out)
        self.stream.synchronize()
        return {k: v.cpu().numpy() for k, v in out.items()}

    def route_baseline_device(self, darr: Optional[DeviceArrivals], out, policy: int, seed: int = 0) -> None:
        """Enqueue one dispatch round of a comparison policy (BR-0 contexts); no synchronisation."""
        a = darr.struct() if darr is not None else None
        o = self.out_struct(out)
        _check(self.lib.br_route_baseline(self.ctx, C.byref(a) if a is not None else None, C.byref(o), int(policy),
                                          int(seed) & (2 ** 64 - 1)), "br_route_baseline", self.ctx)

    def route_baseline(self, arr, policy: int, seed: int = 0):
        """Convenience for tests: host arrays in, numpy out (synchronises)."""
        darr = DeviceArrivals(arr, self.device, 0) if arr is not None else None
        out = self.alloc_outputs(scores=False)
        self.route_baseline_device(darr, out, policy, seed)
        self.stream.synchronize()
        return {k: v.cpu().numpy() for k, v in out.items()}

    def advance(self, n_steps: int = 1) -> None:
        _check(self.lib.br_advance_decode(self.ctx, int(n_steps)), "br_advance_decode", self.ctx)

    def profile(self, on: bool) -> None:
        _check(self.lib.br_profile_enable(self.ctx, int(on)), "br_profile_enable", self.ctx)

    def profile_read(self):
        ms = (C.c_double * NKERNELS)()
        cnt = (C.c_int64 * NKERNELS)()
        _check(self.lib.br_profile_read(self.ctx, ms, cnt), "br_profile_read", self.ctx)
        return {KERNEL_NAMES[k]: (float(ms[k]), int(cnt[k])) for k in range(NKERNELS)}

    # -- state inspection (tests) ----------------------------------------
    def _view(self, off: int, shape, dtype=None):
        torch = self.torch
        n = int(np.prod(shape)) if len(shape) else 1
        v = self.ws[off // 4: off // 4 + n]
        if dtype == "f32":
            v = v.view(torch.float32)
        return v.view(*shape)

    def state(self):
        """Host copies of the snapshot, in the oracle's array shapes (slots beyond n zeroed)."""
        self.stream.synchronize()
        N, G, B, Bs, Q, P, Pq, H = self.N, self.G, self.B, self.Bs, self.Q, self.P, self.Pq, self.H
        lay = self.layout
        st = dict(L=self._view(lay.L, (N, G)).cpu().numpy().astype(np.int64),
                  n=self._view(lay.n, (N, G)).cpu().numpy(),
                  kv=self._view(lay.kv, (N, G, Bs))[:, :, :B].cpu().numpy(),
                  rem=self._view(lay.rem, (N, G, Bs))[:, :, :B].cpu().numpy(),
                  qlen=self._view(lay.qlen, (N,)).cpu().numpy(),
                  qs=self._view(lay.qs, (N, Q)).cpu().numpy(), qo=self._view(lay.qo, (N, Q)).cpu().numpy(),
                  qid=self._view(lay.qid, (N, Q)).cpu().numpy())
        if P:
            st["pred"] = self._view(lay.pred, (N, G, Bs, P), "f32")[:, :, :B].cpu().numpy()
            if Pq:
                st["qpred"] = self._view(lay.qpred, (N, Q, Pq), "f32").cpu().numpy()
        if H > 0:
            st["Lh"] = self._view(lay.Lh, (N, G, H + 1)).cpu().numpy().astype(np.int64)
            st["Mh"] = self._view(lay.Mh, (N, H + 1)).cpu().numpy().astype(np.int64)
            st["mh"] = self._view(lay.mh, (N, G, H + 1)).cpu().numpy().astype(np.int64)
            st["minm"] = self._view(lay.minm, (N, G)).cpu().numpy().astype(np.int64)
        return st

    def close(self) -> None:
        if getattr(self, "ctx", None):
            self.stream.synchronize()
            self.lib.br_free(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
