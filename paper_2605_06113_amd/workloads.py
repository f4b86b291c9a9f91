"""Seeded synthetic inputs for the BalanceRoute route-step path.

This module only draws random cluster snapshots and arrival traces; it holds
none of the routing arithmetic.  Both the CPU oracle tests and the HIP path
tests feed on the arrays produced here, so the two sides always see identical
inputs.  The shapes follow the paper's problem statement (Sec. 2.2: G workers,
slot limit B, prefill length s_i, output length o_i) and the length mixes of
its two evaluation traces (Sec. 6.1: heavy-tailed prompts and outputs); the
records themselves are synthetic.

Array conventions (all little-endian, C-contiguous):
  n    [N][G]        int32  active requests per worker
  kv   [N][G][B]     int32  current KV length of slot j (dense: slots < n[g] used)
  rem  [N][G][B]     int32  remaining decode steps of slot j (>= 1 when used)
  pred [N][G][B][H]  float32 per-step termination hazards of slot j (H > 0 only)
  arrivals per step: count [N] int32, s/o/id [N][arr_cap] int32,
                     pred [N][arr_cap][H] float32
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np

MAX_S = 32768  # largest prefill length any workload here produces


@dataclass(frozen=True)
class RouteConfig:
    """Static parameters of one workload (routing knobs + generator knobs)."""

    name: str
    n_inst: int
    G: int
    B: int
    max_wait: int
    H: int = 0
    R_max: int = 4
    S_greedy: int = -1          # -1 => G * R_max
    token_cap: int = 0
    token_watermark: int = 0
    alpha: float = 1.0
    beta: float = -1.0          # -1 => float(G)
    gamma: float = 0.9
    gate_pfin: float = 0.5
    pred_mode: int = 0          # 0 hazards p[1..H], 1 direct c_hat, 2 empirical-survival estimator, 3 (p_fin, mu_rem)
    refresh_period: int = 0     # pred_mode 2: tokens between predictor refreshes (0 => max(H // 2, 1))
    steps: int = 1
    seed: int = 0
    # generator knobs
    arrival_rate: float = 0.0
    arrival_rate_hi: float = 0.0   # second MMPP state (0 => plain Poisson)
    mmpp_switch: float = 0.0
    prompt_mu: float = float(np.log(1000.0))
    prompt_sigma: float = 1.0
    prompt_lo: int = 16
    prompt_hi: int = 16384
    out_mu: float = float(np.log(200.0))
    out_sigma: float = 1.2
    out_lo: int = 1
    out_hi: int = 4096
    beta_a: float = 2.0
    beta_b: float = 50.0
    init_active_per_worker: int = 0
    init_active_total: int = 0
    init_kv_lo: int = 128
    init_kv_hi: int = 4096
    init_rem_lo: int = 1
    init_rem_hi: int = 512
    init_waiting: int = 0

    @property
    def s_greedy(self) -> int:
        return self.G * self.R_max if self.S_greedy < 0 else self.S_greedy

    @property
    def refresh_eff(self) -> int:
        return self.refresh_period if self.refresh_period > 0 else max(self.H // 2, 1)

    @property
    def beta_eff(self) -> float:
        return float(self.G) if self.beta < 0 else self.beta


def config(name: str, **over) -> RouteConfig:
    """The five workloads (c1..c5) plus small variants used by the tests."""
    base: Dict[str, RouteConfig] = {
        # one BR-0 step, one instance, both stages run
        "c1": RouteConfig(name="c1", n_inst=1, G=4, B=16, max_wait=32, seed=0,
                          token_cap=65536, token_watermark=58982,
                          prompt_hi=8192, init_active_total=20, init_waiting=32),
        # BR-0 replay, overloaded
        "c2": RouteConfig(name="c2", n_inst=1, G=16, B=96, max_wait=256, seed=1000,
                          token_cap=262144, token_watermark=235929, steps=2000,
                          arrival_rate=40.0),
        # BR-H replay, H=4
        "c3": RouteConfig(name="c3", n_inst=1, G=32, B=96, max_wait=512, H=4, seed=2000,
                          token_cap=262144, token_watermark=235929, steps=1000,
                          arrival_rate=80.0, beta_a=2.0, beta_b=50.0),
        # batched BR-0 throughput, token filter off
        "c4": RouteConfig(name="c4", n_inst=4096, G=16, B=144, max_wait=256, seed=3000,
                          init_active_per_worker=128, init_kv_lo=256, init_kv_hi=8192,
                          init_rem_lo=1, init_rem_hi=1024, init_waiting=256),
        # BR-H stress, H=8, bursty arrivals
        "c5": RouteConfig(name="c5", n_inst=1, G=64, B=96, max_wait=2048, H=8, seed=4000,
                          token_cap=524288, token_watermark=471859, steps=10000,
                          arrival_rate=60.0, arrival_rate_hi=300.0, mmpp_switch=1.0 / 200.0,
                          prompt_mu=float(np.log(2000.0)), prompt_sigma=1.1, prompt_hi=32768,
                          out_mu=float(np.log(300.0)), out_sigma=1.3, out_hi=8192,
                          beta_a=2.0, beta_b=40.0),
    }
    cfg = base[name]
    return replace(cfg, **over) if over else cfg


def _lengths(rng: np.random.Generator, mu, sigma, lo, hi, size) -> np.ndarray:
    x = rng.lognormal(mean=mu, sigma=sigma, size=size)
    return np.clip(np.rint(x), lo, hi).astype(np.int32)


def prompts(rng, cfg: RouteConfig, size) -> np.ndarray:
    return _lengths(rng, cfg.prompt_mu, cfg.prompt_sigma, cfg.prompt_lo, cfg.prompt_hi, size)


def outputs(rng, cfg: RouteConfig, size) -> np.ndarray:
    return _lengths(rng, cfg.out_mu, cfg.out_sigma, cfg.out_lo, cfg.out_hi, size)


def hazards(rng, cfg: RouteConfig, size) -> np.ndarray:
    """Per-step termination probabilities of a synthetic classifier (or c_hat draws)."""
    if cfg.H == 0:
        return np.zeros(tuple(np.atleast_1d(size)) + (0,), np.float32)
    if cfg.pred_mode == 1:
        return rng.uniform(0.0, cfg.H + 0.5, size=size).astype(np.float32)
    if cfg.pred_mode == 3:   # a classifier's p_fin (mass at both ends) and a regressor's mu_rem
        shape = tuple(np.atleast_1d(size))
        pf = np.where(rng.random(shape) < 0.5, rng.beta(0.6, 0.6, size=shape), rng.beta(cfg.beta_a, cfg.beta_b, size=shape))
        mu = rng.uniform(0.0, cfg.H + 0.5, size=shape)
        return np.stack([pf, mu], axis=-1).astype(np.float32)
    shape = tuple(np.atleast_1d(size)) + (cfg.H,)
    return rng.beta(cfg.beta_a, cfg.beta_b, size=shape).astype(np.float32)


def informative_hazards(rem: np.ndarray, H: int, hit: float = 0.9, miss: float = 0.02) -> np.ndarray:
    """Hazards of a sharp classifier: high at the true remaining length, low elsewhere."""
    j = np.arange(1, H + 1, dtype=np.int64)
    p = np.where(rem[..., None].astype(np.int64) == j, hit, miss)
    return p.astype(np.float32)


@dataclass
class InitState:
    n: np.ndarray
    kv: np.ndarray
    rem: np.ndarray
    pred: Optional[np.ndarray]


@dataclass
class Arrivals:
    """One batch of arrivals (a single route step) for all instances."""

    count: np.ndarray
    s: np.ndarray
    o: np.ndarray
    id: np.ndarray
    pred: Optional[np.ndarray]

    @property
    def arr_cap(self) -> int:
        return int(self.s.shape[-1])


@dataclass
class Trace:
    """Arrivals for `steps` consecutive route steps: arrays carry a leading step axis."""

    count: np.ndarray            # [steps][N]
    s: np.ndarray                # [steps][N][arr_cap]
    o: np.ndarray
    id: np.ndarray
    pred: Optional[np.ndarray]   # [steps][N][arr_cap][H]
    meta: dict = field(default_factory=dict)

    def step(self, k: int) -> Arrivals:
        return Arrivals(self.count[k], self.s[k], self.o[k], self.id[k],
                        None if self.pred is None else self.pred[k])


def _instance_rngs(cfg: RouteConfig):
    if cfg.n_inst == 1:
        return [np.random.Generator(np.random.PCG64(cfg.seed))]
    kids = np.random.SeedSequence(cfg.seed).spawn(cfg.n_inst)
    return [np.random.Generator(np.random.PCG64(k)) for k in kids]


def slot_pred_width(cfg: RouteConfig) -> int:
    """Floats an ACTIVE request carries: H hazards, one estimate, or (estimate, age, tokens since the last
    query) when the library maintains the estimate itself (pred_mode 2)."""
    if cfg.H == 0:
        return 0
    return {1: 1, 2: 3, 3: 2}.get(cfg.pred_mode, cfg.H)


def maintained_triples(rng, cfg: RouteConfig, size) -> np.ndarray:
    """Initial (estimate, age, tokens since the last query) of requests that are already active when the
    library takes over (pred_mode 2): estimate anywhere in [1, H], a small integer age, a phase below the
    refresh period.  All three are exact in fp32."""
    shape = (size,) if np.isscalar(size) else tuple(size)
    out = np.zeros(shape + (3,), np.float32)
    out[..., 0] = rng.integers(4, 4 * cfg.H + 1, size=shape) / 4.0
    out[..., 1] = rng.integers(0, 40, size=shape)
    out[..., 2] = rng.integers(0, max(cfg.refresh_eff, 1), size=shape)
    return out


def pred_width(cfg: RouteConfig) -> int:
    """Floats a waiting request / an arrival carries for the prediction interface."""
    if cfg.H == 0 or cfg.pred_mode == 2:
        return 0
    return {1: 1, 3: 2}.get(cfg.pred_mode, cfg.H)


def output_history(cfg: RouteConfig, n: int = 4096) -> np.ndarray:
    """Sorted output lengths of a synthetic training corpus (same length mix as the arrivals)."""
    rng = np.random.Generator(np.random.PCG64([cfg.seed, 3]))
    return np.sort(outputs(rng, cfg, n)).astype(np.int32)


def initial_state(cfg: RouteConfig) -> InitState:
    """Active sets at step 0 (dense per-worker lists)."""
    N, G, B, P = cfg.n_inst, cfg.G, cfg.B, slot_pred_width(cfg)
    n = np.zeros((N, G), np.int32)
    kv = np.zeros((N, G, B), np.int32)
    rem = np.zeros((N, G, B), np.int32)
    pred = np.zeros((N, G, B, P), np.float32) if P else None
    slot_pred = (lambda rng, size: maintained_triples(rng, cfg, size)) if cfg.pred_mode == 2 else \
        (lambda rng, size: hazards(rng, cfg, size))
    rngs = _instance_rngs(cfg)
    for i, rng in enumerate(rngs):
        if cfg.init_active_per_worker:
            a = cfg.init_active_per_worker
            n[i, :] = a
            kv[i, :, :a] = rng.integers(cfg.init_kv_lo, cfg.init_kv_hi + 1, size=(G, a))
            rem[i, :, :a] = rng.integers(cfg.init_rem_lo, cfg.init_rem_hi + 1, size=(G, a))
            if P:
                pred[i, :, :a] = slot_pred(rng, (G, a)).reshape(G, a, P)
        elif cfg.init_active_total:
            for _ in range(cfg.init_active_total):
                while True:
                    g = int(rng.integers(0, G))
                    if n[i, g] < B:
                        break
                j = n[i, g]
                kv[i, g, j] = rng.integers(cfg.init_kv_lo, cfg.init_kv_hi + 1)
                rem[i, g, j] = rng.integers(cfg.init_rem_lo, cfg.init_rem_hi + 1)
                if P:
                    pred[i, g, j] = slot_pred(rng, 1).reshape(P)
                n[i, g] += 1
    return InitState(n, kv, rem, pred)


def initial_waiting(cfg: RouteConfig) -> Arrivals:
    """The requests already waiting at step 0 (handed over as the first arrivals)."""
    N, W, P = cfg.n_inst, cfg.init_waiting, pred_width(cfg)
    cap = max(W, 1)
    count = np.full((N,), W, np.int32)
    s = np.zeros((N, cap), np.int32)
    o = np.ones((N, cap), np.int32)
    ids = np.tile(np.arange(cap, dtype=np.int32), (N, 1))
    pred = np.zeros((N, cap, P), np.float32) if P else None
    # a stream separate from initial_state's so the two can be drawn independently
    if N == 1:
        rngs = [np.random.Generator(np.random.PCG64([cfg.seed, 1]))]
    else:
        rngs = [np.random.Generator(np.random.PCG64(k))
                for k in np.random.SeedSequence([cfg.seed, 1]).spawn(N)]
    for i, rng in enumerate(rngs):
        s[i, :W] = prompts(rng, cfg, W)
        o[i, :W] = outputs(rng, cfg, W)
        if P:
            pred[i, :W] = hazards(rng, cfg, W).reshape(W, P)
    return Arrivals(count, s, o, ids, pred)


def arrival_trace(cfg: RouteConfig, steps: Optional[int] = None,
                  informative: bool = False) -> Trace:
    """Arrivals per decode step: Poisson, or 2-state Markov-modulated Poisson."""
    steps = cfg.steps if steps is None else steps
    N, P = cfg.n_inst, pred_width(cfg)
    rng = np.random.Generator(np.random.PCG64([cfg.seed, 2]))
    state = np.zeros((N,), np.int64)
    rates = np.array([cfg.arrival_rate, cfg.arrival_rate_hi or cfg.arrival_rate])
    count = np.zeros((steps, N), np.int32)
    states = np.zeros((steps, N), np.int8)
    for k in range(steps):
        if cfg.mmpp_switch > 0.0:
            flip = rng.random(N) < cfg.mmpp_switch
            state = np.where(flip, 1 - state, state)
        states[k] = state
        count[k] = rng.poisson(rates[state])
    cap = max(int(count.max()), 1)
    s = prompts(rng, cfg, (steps, N, cap))
    o = outputs(rng, cfg, (steps, N, cap))
    pred = None
    if P:
        if informative and cfg.pred_mode == 0:
            pred = informative_hazards(o, cfg.H)
        else:
            pred = hazards(rng, cfg, (steps, N, cap)).reshape(steps, N, cap, P)
    # request ids: running number per instance over the whole trace
    ids = np.zeros((steps, N, cap), np.int32)
    base = np.zeros((N,), np.int64)
    for k in range(steps):
        ids[k] = (base[:, None] + np.arange(cap)[None, :]).astype(np.int32)
        base += count[k]
    return Trace(count, s, o, ids, pred, meta={"mmpp_state": states})


def random_case(seed: int, N: int, G: int, B: int, max_wait: int, H: int = 0,
                fill: float = 0.5, n_wait: Optional[int] = None,
                s_hi: int = 4096, tie_heavy: bool = False, pred_mode: int = 0,
                **cfg_over):
    """A small random snapshot + one batch of arrivals, for property and parity tests.

    `tie_heavy` draws lengths from a tiny alphabet so that equal scores, equal
    loads and equal capacities (the tie-break rules) are exercised.
    """
    rng = np.random.Generator(np.random.PCG64([seed, 77]))
    cfg = RouteConfig(name=f"rand{seed}", n_inst=N, G=G, B=B, max_wait=max_wait, H=H,
                      seed=seed, pred_mode=pred_mode, **cfg_over)
    P = pred_width(cfg)
    n = rng.binomial(B, fill, size=(N, G)).astype(np.int32)
    kv = np.zeros((N, G, B), np.int32)
    rem = np.zeros((N, G, B), np.int32)
    pred = np.zeros((N, G, B, P), np.float32) if P else None
    used = np.arange(B)[None, None, :] < n[:, :, None]
    if tie_heavy:
        kvv = rng.choice(np.array([64, 128, 256], np.int32), size=(N, G, B))
    else:
        kvv = rng.integers(1, s_hi + 1, size=(N, G, B), dtype=np.int32)
    kv[used] = kvv[used]
    remv = rng.integers(1, max(2 * H, 8) + 1, size=(N, G, B), dtype=np.int32)
    rem[used] = remv[used]
    if pred_mode == 2 and H > 0:   # the library maintains the estimate: active requests carry (estimate, age, phase)
        pred = np.zeros((N, G, B, 3), np.float32)
        pred[used] = maintained_triples(rng, cfg, (N, G, B))[used]
    if P:
        pv = hazards(rng, cfg, (N, G, B)).reshape(N, G, B, P)
        if pred_mode == 0:
            # mix in sharp hazards so the in-window cut-off branch is live
            sharp = informative_hazards(remv, H)
            pick = rng.random((N, G, B)) < 0.5
            pv = np.where(pick[..., None], sharp, pv).astype(np.float32)
        pred[used] = pv[used]
    W = max_wait if n_wait is None else n_wait
    cap = max(W, 1)
    count = rng.integers(0, W + 1, size=(N,), dtype=np.int32) if n_wait is None \
        else np.full((N,), W, np.int32)
    if tie_heavy:
        s = rng.choice(np.array([64, 128, 192, 256], np.int32), size=(N, cap))
    else:
        s = rng.integers(1, s_hi + 1, size=(N, cap), dtype=np.int32)
    o = rng.integers(1, 64, size=(N, cap), dtype=np.int32)
    ids = rng.integers(0, 2 ** 30, size=(N, cap), dtype=np.int32)
    apred = hazards(rng, cfg, (N, cap)).reshape(N, cap, P) if P else None
    return cfg, InitState(n, kv, rem, pred), Arrivals(count, s, o, ids, apred)
