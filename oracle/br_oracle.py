"""ctypes front end of the BalanceRoute CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
module.  It marshals numpy arrays into oracle/br_oracle.c; the arithmetic all
lives in the C file.  Nothing here touches the GPU library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "br_oracle.c")
_HDR = os.path.join(_HERE, "br_oracle.h")
_LIB = os.path.join(_HERE, "libbr_oracle.so")

NSTATS = 16
ST = dict(admitted=0, deferred=1, dropped=2, stage1=3, stage2_pops=4, guard=5, overcap=6,
          I_before=7, I_after=8, spread=9, qlen=10, workers_dropped=11, load_range=12)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no contraction, no fast-math)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_HDR)))
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-Wall",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Params(C.Structure):
    _fields_ = [("G", C.c_int32), ("B", C.c_int32), ("max_wait", C.c_int32), ("H", C.c_int32),
                ("R_max", C.c_int32), ("S_greedy", C.c_int32),
                ("token_watermark", C.c_int32), ("token_cap", C.c_int32),
                ("pred_mode", C.c_int32), ("force_float", C.c_int32),
                ("alpha", C.c_float), ("beta", C.c_float), ("gamma", C.c_float),
                ("gate_pfin", C.c_float),
                ("hist", C.c_void_p), ("hist_sum", C.c_void_p), ("hist_n", C.c_int32), ("refresh", C.c_int32)]


class Event(C.Structure):
    _fields_ = [("g", C.c_int32), ("stage", C.c_int32), ("n_req", C.c_int32), ("pad", C.c_int32),
                ("delta", C.c_int64), ("score", C.c_double)]


_P = C.c_void_p


class IO(C.Structure):
    _fields_ = [("L", _P), ("n", _P), ("kv", _P), ("rem", _P), ("pred", _P),
                ("qlen", _P), ("qs", _P), ("qo", _P), ("qid", _P), ("qpred", _P),
                ("a_count", C.c_int32), ("pad0", C.c_int32),
                ("a_s", _P), ("a_o", _P), ("a_id", _P), ("a_pred", _P),
                ("assign", _P), ("assign_id", _P), ("stats", _P), ("F_i32", _P), ("F_f32", _P),
                ("best_g", _P), ("best_i", _P), ("Lh", _P), ("Mh", _P), ("mh", _P), ("minm", _P),
                ("chat", _P), ("events", _P), ("n_events", _P)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        # BR_ORACLE_LIB: a build of this oracle to load instead (the mutation test points it at copies of
        # br_oracle.c with one planted mistake each, to show that the pins notice)
        _lib = C.CDLL(os.environ.get("BR_ORACLE_LIB") or build())
        _lib.orc_score_br0.restype = C.c_int64
        _lib.orc_score_br0.argtypes = [C.c_int64, C.c_int64, C.c_int64]
        _lib.orc_score_brh.restype = C.c_float
        _lib.orc_score_brh.argtypes = [C.c_int32, C.c_float, C.c_float, C.c_float, _P, C.c_int64]
        _lib.orc_chat.restype = C.c_float
        _lib.orc_chat.argtypes = [C.c_int32, C.c_int32, C.c_float, _P]
        _lib.orc_best_subset.restype = C.c_int32
        _lib.orc_best_subset.argtypes = [C.POINTER(Params), _P, C.c_int64, C.c_int32, _P, C.c_int32,
                                         C.POINTER(C.c_double)]
        _lib.orc_best_subset_reach.restype = C.c_int32
        _lib.orc_best_subset_reach.argtypes = _lib.orc_best_subset.argtypes
        for f in (_lib.orc_project, _lib.orc_route_step, _lib.orc_route_bypass):
            f.restype = C.c_int32
            f.argtypes = [C.POINTER(Params), C.POINTER(IO)]
        _lib.orc_hash64.restype = C.c_uint64
        _lib.orc_hash64.argtypes = [C.c_uint64, C.c_uint64]
        _lib.orc_route_baseline.restype = C.c_int32
        _lib.orc_route_baseline.argtypes = [C.POINTER(Params), C.POINTER(IO), C.c_int32, C.c_uint64, C.c_int32, _P]
        _lib.orc_advance.restype = C.c_int32
        _lib.orc_advance.argtypes = [C.POINTER(Params), C.POINTER(IO), C.c_int32]
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_P)


POLICY = dict(random=0, rr=1, p2c=2, jsq=3)


def hash64(key: int, c: int) -> int:
    return int(lib().orc_hash64(key & (2 ** 64 - 1), c))


def score_br0(G: int, m: int, delta: int) -> int:
    return int(lib().orc_score_br0(G, m, delta))


def score_brh(H: int, alpha: float, beta: float, gamma: float, m, delta: int) -> float:
    mm = np.ascontiguousarray(m, np.int64)
    assert mm.shape == (H + 1,)
    return float(lib().orc_score_brh(H, alpha, beta, gamma, _ptr(mm), int(delta)))


def chat(H: int, pred_mode: int, gate_pfin: float, p) -> float:
    pp = np.ascontiguousarray(p, np.float32)
    return float(lib().orc_chat(H, pred_mode, gate_pfin, _ptr(pp)))


def params_from(cfg, force_float: bool = False, hist=None) -> Params:
    """cfg: any object with the RouteConfig fields; hist: sorted output-length history (pred_mode 2).
    The returned struct keeps the history arrays alive in `_keep`."""
    P = Params(G=cfg.G, B=cfg.B, max_wait=cfg.max_wait, H=cfg.H, R_max=cfg.R_max,
               S_greedy=cfg.s_greedy, token_watermark=cfg.token_watermark,
               token_cap=cfg.token_cap, pred_mode=cfg.pred_mode, force_float=int(force_float),
               alpha=cfg.alpha, beta=cfg.beta_eff, gamma=cfg.gamma, gate_pfin=cfg.gate_pfin,
               hist=None, hist_sum=None, hist_n=0, refresh=int(getattr(cfg, "refresh_eff", 1)))
    if hist is not None:
        h = np.ascontiguousarray(hist, np.int32)
        assert (np.diff(h) >= 0).all(), "history must be sorted"
        hs = np.concatenate([[0], np.cumsum(h, dtype=np.int64)]).astype(np.int64)
        P._keep = (h, hs)
        P.hist, P.hist_sum, P.hist_n = h.ctypes.data, hs.ctypes.data, len(h)
    return P


def survival(params: Params, age: int) -> float:
    lib().orc_survival.restype = C.c_float
    lib().orc_survival.argtypes = [C.POINTER(Params), C.c_int64]
    return float(lib().orc_survival(C.byref(params), int(age)))


def best_subset(params: Params, m_g, L_g: int, cap_g: int, win_s):
    mm = np.ascontiguousarray(m_g, np.int64)
    ws = np.ascontiguousarray(win_s, np.int32)
    f = C.c_double(0.0)
    mask = lib().orc_best_subset(C.byref(params), _ptr(mm), int(L_g), int(cap_g), _ptr(ws), len(ws),
                                 C.byref(f))
    return int(mask), float(f.value)


def best_subset_reach(params: Params, m_g, L_g: int, cap_g: int, win_s):
    """The subset search by reachable sums (any window up to 32 requests); mask as an unsigned 32-bit value."""
    mm = np.ascontiguousarray(m_g, np.int64)
    ws = np.ascontiguousarray(win_s, np.int32)
    f = C.c_double(0.0)
    mask = lib().orc_best_subset_reach(C.byref(params), _ptr(mm), int(L_g), int(cap_g), _ptr(ws), len(ws),
                                       C.byref(f))
    return int(mask) & 0xFFFFFFFF, float(f.value)


class OracleCluster:
    """N independent instances held as numpy arrays; every call loops over them in C."""

    def __init__(self, cfg, init=None, force_float: bool = False, hist=None):
        self.cfg = cfg
        self.params = params_from(cfg, force_float, hist)
        N, G, B, Q, H = cfg.n_inst, cfg.G, cfg.B, cfg.max_wait, cfg.H
        self.N, self.G, self.B, self.Q, self.H = N, G, B, Q, H
        self.P = 0 if H == 0 else {1: 1, 2: 3, 3: 2}.get(cfg.pred_mode, H)
        self.Pq = 0 if cfg.pred_mode == 2 else self.P
        self.use_float = H > 0 or force_float
        self.L = np.zeros((N, G), np.int64)
        self.n = np.zeros((N, G), np.int32)
        self.kv = np.zeros((N, G, B), np.int32)
        self.rem = np.zeros((N, G, B), np.int32)
        self.pred = np.zeros((N, G, B, self.P), np.float32) if self.P else None
        self.qlen = np.zeros((N,), np.int32)
        self.qs = np.zeros((N, Q), np.int32)
        self.qo = np.zeros((N, Q), np.int32)
        self.qid = np.zeros((N, Q), np.int32)
        self.qpred = np.zeros((N, Q, self.Pq), np.float32) if self.Pq else None
        if init is not None:
            self.n[...] = init.n
            self.kv[...] = init.kv
            self.rem[...] = init.rem
            if self.P:
                if init.pred is None:
                    assert not np.any(init.n), "active requests need their prediction rows"
                else:
                    assert np.shape(init.pred) == self.pred.shape, "init.pred: wrong shape"
                    self.pred[...] = init.pred
            used = np.arange(B)[None, None, :] < self.n[:, :, None]
            self.kv[~used] = 0
            self.rem[~used] = 0
            self.L[...] = np.where(used, self.kv, 0).sum(axis=2)

    # -- helpers -------------------------------------------------------
    def _io(self, i: int) -> IO:
        io = IO()
        io.L, io.n, io.kv, io.rem = _ptr(self.L[i]), _ptr(self.n[i]), _ptr(self.kv[i]), _ptr(self.rem[i])
        io.pred = _ptr(self.pred[i]) if self.P else None
        io.qlen = _ptr(self.qlen[i:i + 1])
        io.qs, io.qo, io.qid = _ptr(self.qs[i]), _ptr(self.qo[i]), _ptr(self.qid[i])
        io.qpred = _ptr(self.qpred[i]) if self.Pq else None
        return io

    def project(self):
        """Projected loads, envelope, margins and c_hat of the current active sets."""
        N, G, B, H = self.N, self.G, self.B, self.H
        out = dict(Lh=np.zeros((N, G, H + 1), np.int64), Mh=np.zeros((N, H + 1), np.int64),
                   mh=np.zeros((N, G, H + 1), np.int64), minm=np.zeros((N, G), np.int64),
                   chat=np.zeros((N, G, B), np.float32))
        for i in range(N):
            io = self._io(i)
            io.Lh, io.Mh, io.mh, io.minm, io.chat = (_ptr(out["Lh"][i]), _ptr(out["Mh"][i]),
                                                      _ptr(out["mh"][i]), _ptr(out["minm"][i]),
                                                      _ptr(out["chat"][i]))
            rc = lib().orc_project(C.byref(self.params), C.byref(io))
            assert rc == 0
        return out

    def route_step(self, arr=None, want_scores: bool = True, want_events: bool = False,
                   want_prep: bool = False):
        """One routing round on every instance.  `arr` is a workloads.Arrivals or None."""
        N, G, B, Q, H = self.N, self.G, self.B, self.Q, self.H
        out = dict(assign=np.full((N, Q), -1, np.int32), assign_id=np.full((N, Q), -1, np.int32),
                   stats=np.zeros((N, NSTATS), np.int64))
        if want_scores:
            out["F"] = np.zeros((N, Q, G), np.float32 if self.use_float else np.int32)
            out["best_g"] = np.full((N, Q), -1, np.int32)
            out["best_i"] = np.full((N, G), -1, np.int32)
        if want_prep:
            out.update(Lh=np.zeros((N, G, H + 1), np.int64), Mh=np.zeros((N, H + 1), np.int64),
                       mh=np.zeros((N, G, H + 1), np.int64), minm=np.zeros((N, G), np.int64))
        if want_events:
            ev = np.zeros((N, Q), dtype=np.dtype([("g", "<i4"), ("stage", "<i4"), ("n_req", "<i4"),
                                                  ("pad", "<i4"), ("delta", "<i8"), ("score", "<f8")]))
            nev = np.zeros((N,), np.int32)
            out["events"], out["n_events"] = ev, nev
        if arr is not None:
            a_s = np.ascontiguousarray(arr.s, np.int32)
            a_o = np.ascontiguousarray(arr.o, np.int32)
            a_id = np.ascontiguousarray(arr.id, np.int32)
            a_pred = np.ascontiguousarray(arr.pred, np.float32) if self.Pq else None
        for i in range(N):
            io = self._io(i)
            if arr is not None:
                io.a_count = int(arr.count[i])
                io.a_s, io.a_o, io.a_id = _ptr(a_s[i]), _ptr(a_o[i]), _ptr(a_id[i])
                io.a_pred = _ptr(a_pred[i]) if self.Pq else None
            io.assign, io.assign_id, io.stats = (_ptr(out["assign"][i]), _ptr(out["assign_id"][i]),
                                                 _ptr(out["stats"][i]))
            if want_scores:
                if self.use_float:
                    io.F_f32 = _ptr(out["F"][i])
                else:
                    io.F_i32 = _ptr(out["F"][i])
                io.best_g, io.best_i = _ptr(out["best_g"][i]), _ptr(out["best_i"][i])
            if want_prep:
                io.Lh, io.Mh, io.mh, io.minm = (_ptr(out["Lh"][i]), _ptr(out["Mh"][i]),
                                                _ptr(out["mh"][i]), _ptr(out["minm"][i]))
            if want_events:
                io.events, io.n_events = _ptr(out["events"][i]), _ptr(out["n_events"][i:i + 1])
            rc = lib().orc_route_step(C.byref(self.params), C.byref(io))
            assert rc == 0, rc
        return out

    def route_bypass(self, arr):
        """Pool-bypass dispatch of one batch of arrivals (BR-0 only); assign is per arrival."""
        N = self.N
        cap = int(arr.s.shape[-1])
        out = dict(assign=np.full((N, cap), -3, np.int32), stats=np.zeros((N, NSTATS), np.int64))
        a_s = np.ascontiguousarray(arr.s, np.int32)
        a_o = np.ascontiguousarray(arr.o, np.int32)
        a_id = np.ascontiguousarray(arr.id, np.int32)
        for i in range(N):
            io = self._io(i)
            io.a_count = int(min(max(arr.count[i], 0), cap))
            io.a_s, io.a_o, io.a_id = _ptr(a_s[i]), _ptr(a_o[i]), _ptr(a_id[i])
            io.assign, io.stats = _ptr(out["assign"][i]), _ptr(out["stats"][i])
            rc = lib().orc_route_bypass(C.byref(self.params), C.byref(io))
            assert rc == 0, rc
        return out

    def route_baseline(self, arr, policy: int, seed: int = 0):
        """One dispatch round of a comparison policy (BR-0 contexts): FIFO over the waiting queue."""
        N, Q = self.N, self.Q
        if not hasattr(self, "pol_state"):
            self.pol_state = np.zeros((N, 2), np.int32)     # round-robin cursor, draws made
        out = dict(assign=np.full((N, Q), -1, np.int32), assign_id=np.full((N, Q), -1, np.int32),
                   stats=np.zeros((N, NSTATS), np.int64))
        if arr is not None:
            a_s = np.ascontiguousarray(arr.s, np.int32)
            a_o = np.ascontiguousarray(arr.o, np.int32)
            a_id = np.ascontiguousarray(arr.id, np.int32)
        for i in range(N):
            io = self._io(i)
            if arr is not None:
                io.a_count = int(arr.count[i])
                io.a_s, io.a_o, io.a_id = _ptr(a_s[i]), _ptr(a_o[i]), _ptr(a_id[i])
            io.assign, io.assign_id, io.stats = (_ptr(out["assign"][i]), _ptr(out["assign_id"][i]),
                                                 _ptr(out["stats"][i]))
            rc = lib().orc_route_baseline(C.byref(self.params), C.byref(io), int(policy), int(seed) & (2 ** 64 - 1), i,
                                          _ptr(self.pol_state[i]))
            assert rc == 0, rc
        return out

    def advance(self, n_steps: int = 1):
        for i in range(self.N):
            io = self._io(i)
            rc = lib().orc_advance(C.byref(self.params), C.byref(io), int(n_steps))
            assert rc == 0

    def snapshot(self):
        return dict(L=self.L.copy(), n=self.n.copy(), kv=self.kv.copy(), rem=self.rem.copy(),
                    pred=None if self.pred is None else self.pred.copy(),
                    qlen=self.qlen.copy(), qs=self.qs.copy(), qo=self.qo.copy(), qid=self.qid.copy(),
                    qpred=None if self.qpred is None else self.qpred.copy())
