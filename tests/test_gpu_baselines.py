"""The comparison policies (Sec. 6.1 "Baselines": Random, RR, P2C, JSQ) through the C ABI against the CPU oracle,
and the quality replay: trace-mean imbalance (max - min load per step, Sec. 6.1 "Metrics") of every policy next to
BR-0 and BR-H on the same synthetic trace, every step of every policy checked against the oracle, with the paper's
qualitative ordering (Sec. 6.2: every BalanceRoute row below every baseline row) asserted on the result."""
import dataclasses
import sys

import numpy as np
import pytest

from oracle import br_oracle
from paper_2605_06113_amd import binding, workloads as wl
from tests.parity import compare_outputs, compare_state

pytestmark = pytest.mark.gpu
POLICIES = ("random", "rr", "p2c", "jsq")


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("G,B,Q,N,fill", [(4, 8, 32, 5, 0.5), (16, 24, 256, 6, 0.8), (64, 12, 2048, 2, 0.3), (1, 5, 17, 3, 0.2),
                                         (33, 40, 700, 3, 0.95), (7, 3, 300, 300, 0.0), (64, 1024, 64, 2, 0.99)])
def test_policies_match_oracle(G, B, Q, N, fill):
    for policy in POLICIES:
        _say(f"policy {policy}: G={G} B={B} Q={Q} N={N}")
        cfg, init, arr = wl.random_case(40 + G + Q, N=N, G=G, B=B, max_wait=Q, H=0, fill=fill, s_hi=32768)
        oc, r = br_oracle.OracleCluster(cfg, init), binding.Router(cfg, init)
        for rnd in range(4):
            if rnd:
                _, _, arr = wl.random_case(140 + G + Q + rnd, N=N, G=G, B=B, max_wait=Q, H=0, n_wait=max(1, Q // (2 * rnd)))
            a = None if rnd == 3 else arr                                   # last round: no arrivals at all
            ref = oc.route_baseline(a, br_oracle.POLICY[policy], seed=1234 + rnd)
            out = r.route_baseline(a, binding.POLICY[policy], seed=1234 + rnd)
            compare_outputs(ref, out, cfg, f"{policy} r{rnd}")
            compare_state(oc, r.state(), cfg, f"{policy} r{rnd}")
            oc.advance(2), r.advance(2)
            compare_state(oc, r.state(), cfg, f"{policy} r{rnd} advanced")
        # a scheduling round of BR-0 afterwards works on the same state
        compare_outputs(oc.route_step(arr), r.route_step(arr), cfg, f"{policy} then BR-0")
        compare_state(oc, r.state(), cfg, f"{policy} then BR-0")
        r.close()


def test_policy_rejects_horizon_contexts_and_unknown_policies():
    import ctypes as C
    cfg, init, arr = wl.random_case(3, N=2, G=4, B=8, max_wait=32, H=4, gate_pfin=0.0)
    r = binding.Router(cfg, init)
    o = r.out_struct(r.alloc_outputs(scores=False))
    assert r.lib.br_route_baseline(r.ctx, None, C.byref(o), 0, 0) == binding.BR_EINVAL
    r.close()
    cfg, init, arr = wl.random_case(3, N=2, G=4, B=8, max_wait=32, H=0)
    r = binding.Router(cfg, init)
    o = r.out_struct(r.alloc_outputs(scores=False))
    assert r.lib.br_route_baseline(r.ctx, None, C.byref(o), 4, 0) == binding.BR_EINVAL
    assert r.lib.br_route_baseline(r.ctx, None, C.byref(o), -1, 0) == binding.BR_EINVAL
    r.close()


def _replay(cfg, policy, steps, oracle_estimate=False, seed=5):
    """One policy over one trace on both sides; returns the per-step spread after each round (GPU's, equal to
    the oracle's).  oracle_estimate: the caller keeps c_hat = min(remaining steps, H) in the workspace (the
    paper's "BR-H oracle" configuration, Sec. 6.1), as a proxy that knows the trace would."""
    tr = wl.arrival_trace(cfg, steps)
    oc, r = br_oracle.OracleCluster(cfg), binding.Router(cfg)
    out = r.alloc_outputs(scores=False)
    lay = r.layout
    spread = np.zeros(steps, np.int64)
    for k in range(steps):
        a = tr.step(k)
        if oracle_estimate:
            a = wl.Arrivals(a.count, a.s, a.o, a.id, np.minimum(a.o, cfg.H).astype(np.float32)[..., None])
        darr = binding.DeviceArrivals(a, r.device, r.Pq)
        if policy in binding.POLICY:
            ref = oc.route_baseline(a, br_oracle.POLICY[policy], seed)
            r.route_baseline_device(darr, out, binding.POLICY[policy], seed)
        else:
            ref = oc.route_step(a, want_scores=False)
            r.route_step_device(darr, out)
        r.advance(1)
        oc.advance(1)
        if oracle_estimate:       # the estimate follows the true remaining length on both sides
            oc.pred[..., 0] = np.minimum(oc.rem, cfg.H)
            oc.qpred[..., 0] = np.minimum(oc.qo, cfg.H)
            pv = r._view(lay.pred, (r.N, r.G, r.Bs, 1), "f32")
            pv[..., 0].copy_(r._view(lay.rem, (r.N, r.G, r.Bs)).clamp(max=cfg.H).float())
            qv = r._view(lay.qpred, (r.N, r.Q, 1), "f32")
            qv[..., 0].copy_(r._view(lay.qo, (r.N, r.Q)).clamp(max=cfg.H).float())
        r.stream.synchronize()
        got = {kk: out[kk].cpu().numpy() for kk in ("assign", "assign_id", "stats")}
        compare_outputs(ref, got, cfg, f"{policy} step {k}")
        spread[k] = got["stats"][0, binding.ST["spread"]]
        if k % 200 == 0 or k == steps - 1:
            compare_state(oc, r.state(), cfg, f"{policy} step {k}")
    r.close()
    return spread


@pytest.mark.parametrize("name,steps,over", [("c2", 2000, {}), ("c3", 1000, {}), ("c5", 1500, {})])
def test_quality_replay_ordering(name, steps, over):
    """Trace-mean imbalance per policy on the replay workloads (the shapes of c2 / c3 / c5; comparison policies
    and BR-0 on the H = 0 context of that shape, BR-H with the true remaining lengths as estimate).  Synthetic
    traces: the ordering is the paper's qualitative result, the figures are not its numbers."""
    base = wl.config(name, token_watermark=0, token_cap=0, **over)
    H = base.H if base.H > 0 else 8
    flat = dataclasses.replace(base, H=0, pred_mode=0)
    mean = {}
    for policy in POLICIES + ("br0",):
        _say(f"quality {name}: {policy}")
        sp = _replay(flat, policy, steps)
        mean[policy] = float(sp[steps // 5:].mean())          # after the warm-up fifth
    _say(f"quality {name}: brh (H={H}, true remaining lengths)")
    mean["brh"] = float(_replay(dataclasses.replace(base, H=H, pred_mode=1), "brh", steps, oracle_estimate=True)[steps // 5:].mean())
    _say(f"quality {name}: " + ", ".join(f"{k} {v:.0f}" for k, v in mean.items()))
    worst_br = max(mean["br0"], mean["brh"])
    assert all(worst_br < mean[p] for p in POLICIES), mean      # every BalanceRoute row below every baseline row
    assert mean["br0"] < 0.7 * min(mean[p] for p in POLICIES), mean
    assert mean["brh"] < mean["br0"], mean                      # lookahead with perfect prediction tightens it further
