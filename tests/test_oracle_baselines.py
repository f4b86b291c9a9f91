"""Pins for the oracle's comparison policies (Sec. 6.1 "Baselines": Random, Round-Robin, Power-of-Two-Choices,
Join-Shortest-Queue): the generator against its published outputs, hand-worked dispatch sequences, structural
properties (arrival order, slot limit, conservation) and the uniformity of the random picks."""
import os

import numpy as np
import pytest

from paper_2605_06113_amd import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))


def _cluster(orc, n, B, G=None, kv=100, max_wait=64):
    G = len(n) if G is None else G
    cfg = wl.RouteConfig(name="pol", n_inst=1, G=G, B=B, max_wait=max_wait, H=0)
    st = wl.InitState(np.array([n], np.int32), np.zeros((1, G, B), np.int32), np.zeros((1, G, B), np.int32), None)
    for g, c in enumerate(n):
        st.kv[0, g, :c] = kv
        st.rem[0, g, :c] = 50
    return cfg, orc.OracleCluster(cfg, st)


def _arr(s):
    s = np.asarray(s, np.int32)[None, :]
    n = s.shape[1]
    return wl.Arrivals(np.array([n], np.int32), s, np.full((1, n), 5, np.int32), np.arange(n, dtype=np.int32)[None, :], None)


def test_generator_matches_published_outputs(orc):
    want = [int(line, 16) for line in open(os.path.join(HERE, "golden", "splitmix64_seed0.txt")) if not line.startswith("#")]
    assert [orc.hash64(0, c) for c in range(3)] == want
    # counter-based: draw c of the stream started at `key` is output c of SplitMix64 seeded with key, so a stream
    # started one increment later is the same stream shifted by one
    assert orc.hash64(0x9E3779B97F4A7C15, 0) == want[1] and orc.hash64(2 * 0x9E3779B97F4A7C15 % 2 ** 64, 0) == want[2]


def test_round_robin_hand_worked(orc):
    cfg, oc = _cluster(orc, [0, 0, 0], B=3)
    out = oc.route_baseline(_arr([10, 20, 30, 40, 50]), orc.POLICY["rr"])
    assert out["assign"][0, :5].tolist() == [0, 1, 2, 0, 1]
    assert oc.L[0].tolist() == [50, 70, 30] and oc.n[0].tolist() == [2, 2, 1]
    # the cursor persists across calls: the next request goes to worker 2
    out = oc.route_baseline(_arr([7]), orc.POLICY["rr"])
    assert out["assign"][0, 0] == 2
    # a full worker is skipped: cursor at 0, worker 1 full
    cfg, oc = _cluster(orc, [0, 2, 0], B=2)
    out = oc.route_baseline(_arr([1, 2, 3, 4, 5]), orc.POLICY["rr"])
    assert out["assign"][0, :5].tolist() == [0, 2, 0, 2, -1]           # four free slots: the fifth keeps waiting
    st = out["stats"][0]
    assert st[orc.ST["admitted"]] == 4 and st[orc.ST["deferred"]] == 1 and oc.qlen[0] == 1 and oc.qs[0, 0] == 5


def test_join_shortest_queue_hand_worked(orc):
    # counts (2, 1, 1): lowest index among the emptiest -> 1; then (2, 2, 1) -> 2; then all 2 -> 0, 1, 2 in turn
    cfg, oc = _cluster(orc, [2, 1, 1], B=4)
    out = oc.route_baseline(_arr([500, 9, 9, 9, 9, 9]), orc.POLICY["jsq"])
    assert out["assign"][0, :6].tolist() == [1, 2, 0, 1, 2, 0]
    # lengths play no role: the 500-token request went to the emptiest worker although it is not the lightest
    assert oc.L[0].tolist() == [200 + 9 + 9, 100 + 500 + 9, 100 + 9 + 9]


def test_random_and_p2c_hand_worked_from_the_published_draws(orc):
    # seed 0, cluster 0: draw 0 = 0xE220A839_7B1DCDAF, draw 1 = 0x6E789E6A_A1B965F4.
    # Four eligible workers: low half 0x7B1DCDAF * 4 >> 32 = 1 -> worker 1; draw 1: 0xA1B965F4 * 4 >> 32 = 2.
    cfg, oc = _cluster(orc, [0, 0, 0, 0], B=8)
    out = oc.route_baseline(_arr([5, 5]), orc.POLICY["random"], seed=0)
    assert out["assign"][0, :2].tolist() == [1, 2]
    # P2C, draw 0: first pick worker 1; high half 0xE220A839 * 3 >> 32 = 2 -> third of the others (0, 2, 3) = 3
    for counts, want in (([0, 5, 0, 2], 3), ([0, 2, 0, 5], 1), ([0, 3, 0, 3], 1)):
        cfg, oc = _cluster(orc, counts, B=8)
        assert oc.route_baseline(_arr([5]), orc.POLICY["p2c"], seed=0)["assign"][0, 0] == want
    # worker 1 full: three eligible (0, 2, 3): 0x7B1DCDAF * 3 >> 32 = 1 -> worker 2; 0xE220A839 * 2 >> 32 = 1 -> second of (0, 3) = 3
    cfg, oc = _cluster(orc, [4, 8, 1, 6], B=8)
    assert oc.route_baseline(_arr([5]), orc.POLICY["p2c"], seed=0)["assign"][0, 0] == 2
    cfg, oc = _cluster(orc, [4, 8, 7, 6], B=8)
    assert oc.route_baseline(_arr([5]), orc.POLICY["p2c"], seed=0)["assign"][0, 0] == 3
    # one eligible worker: it takes the request whatever the draw
    cfg, oc = _cluster(orc, [8, 8, 3, 8], B=8)
    assert oc.route_baseline(_arr([5]), orc.POLICY["p2c"], seed=0)["assign"][0, 0] == 2


@pytest.mark.parametrize("policy", ["random", "rr", "p2c", "jsq"])
def test_structure_of_a_dispatch_round(orc, policy):
    """Arrival order, slot limit, conservation of load and requests, queue cap."""
    rng = np.random.default_rng(3)
    for case in range(30):
        G, B, Q = int(rng.integers(1, 9)), int(rng.integers(1, 7)), 24
        cfg, init, arr = wl.random_case(900 + case, N=3, G=G, B=B, max_wait=Q, H=0, fill=float(rng.choice([0.0, 0.5, 0.9])))
        oc = orc.OracleCluster(cfg, init)
        for rnd in range(3):
            before = oc.snapshot()
            out = oc.route_baseline(arr, orc.POLICY[policy], seed=case)
            for i in range(3):
                qn = int(out["stats"][i, orc.ST["qlen"]])
                free = int((B - before["n"][i]).sum())
                k = min(free, qn)
                a = out["assign"][i]
                assert (a[:k] >= 0).all() and (a[k:] == -1).all()                 # a prefix in arrival order
                assert out["stats"][i, orc.ST["admitted"]] == k and oc.qlen[i] == qn - k
                assert (oc.n[i] <= B).all() and oc.n[i].sum() == before["n"][i].sum() + k
                s_all = np.concatenate([before["qs"][i, :before["qlen"][i]], np.clip(arr.s[i], 1, 32768)])[:qn]
                for g in range(G):
                    assert oc.L[i, g] == before["L"][i, g] + s_all[:k][a[:k] == g].sum()
                assert np.array_equal(oc.qs[i, :qn - k], s_all[k:])
                used = np.arange(B)[None, :] < oc.n[i][:, None]
                assert (np.where(used, oc.kv[i], 0).sum(axis=1) == oc.L[i]).all()
            oc.advance(2)


def test_random_picks_are_uniform_and_p2c_prefers_the_emptier(orc):
    G, B = 8, 4096
    cfg, oc = _cluster(orc, [0] * G, B=B, max_wait=2048)
    counts = np.zeros(G)
    for rnd in range(10):
        out = oc.route_baseline(_arr(np.ones(2048, np.int32)), orc.POLICY["random"], seed=12345)
        counts += np.bincount(out["assign"][0], minlength=G)
    n = counts.sum()
    assert n == 20480 and np.abs(counts - n / G).max() < 5 * np.sqrt(n / G)      # within five sigma of uniform
    # two workers, P2C: both are always drawn, so the emptier one always gets the request
    cfg, oc = _cluster(orc, [30, 10], B=64)
    out = oc.route_baseline(_arr(np.ones(20, np.int32)), orc.POLICY["p2c"], seed=9)
    assert out["assign"][0, :20].tolist() == [1] * 20
    # many workers: P2C's counts stay tighter than Random's (the point of the second choice)
    spread = {}
    for pol in ("random", "p2c"):
        cfg, oc = _cluster(orc, [0] * 16, B=4096, G=16, max_wait=2048)
        for rnd in range(4):
            oc.route_baseline(_arr(np.ones(2048, np.int32)), orc.POLICY[pol], seed=77)
        spread[pol] = int(oc.n[0].max() - oc.n[0].min())
    assert spread["p2c"] < spread["random"]


def test_quality_ordering_on_the_replay_workload(orc):
    """Trace-mean imbalance (max - min load per step, Sec. 6.1 "Metrics") of every policy on the c2 replay
    (synthetic trace: the ordering is the paper's qualitative result of Sec. 6.2, the figures are not its numbers):
    BR-H with the true remaining lengths as estimate < BR-0 < every comparison policy."""
    import dataclasses
    base = wl.config("c2", token_watermark=0, token_cap=0)
    steps = 1200
    tr = wl.arrival_trace(base, steps)
    mean = {}
    for policy in ("random", "rr", "p2c", "jsq", "br0", "brh"):
        cfg = dataclasses.replace(base, H=8, pred_mode=1) if policy == "brh" else base
        oc = orc.OracleCluster(cfg)
        sp = []
        for k in range(steps):
            a = tr.step(k)
            if policy == "brh":
                a = wl.Arrivals(a.count, a.s, a.o, a.id, np.minimum(a.o, cfg.H).astype(np.float32)[..., None])
                out = oc.route_step(a, want_scores=False)
            elif policy == "br0":
                out = oc.route_step(a, want_scores=False)
            else:
                out = oc.route_baseline(a, orc.POLICY[policy], seed=5)
            sp.append(int(out["stats"][0, orc.ST["spread"]]))
            oc.advance(1)
            if policy == "brh":      # a proxy that knows the trace keeps c_hat = min(remaining steps, H)
                oc.pred[..., 0] = np.minimum(oc.rem, cfg.H)
                oc.qpred[..., 0] = np.minimum(oc.qo, cfg.H)
        mean[policy] = float(np.mean(sp[steps // 5:]))
    assert mean["brh"] < mean["br0"] < 0.7 * min(mean[p] for p in ("random", "rr", "p2c", "jsq")), mean
