"""Parity of the HIP path (called through the C ABI) against the CPU oracle, element by element
on the same seeded inputs.  Integer results (assignments, loads, slot tables, queue, BR-0 scores,
statistics) must be bit-exact; fp32 horizon scores within 1e-5 relative."""
import sys

import numpy as np
import pytest

from oracle import br_oracle
from paper_2605_06113_amd import binding, workloads as wl
from tests.parity import compare_outputs, compare_prep, compare_state, run_pair

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def test_c1_single_step():
    cfg = wl.config("c1")
    _say("c1")
    oc, r = run_pair(cfg, wl.initial_state(cfg), wl.initial_waiting(cfg), tag="c1")
    r.close()
    # and against the stored result of the oracle (tests/golden/c1_round.txt)
    import os
    gold = {}
    for line in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "c1_round.txt")):
        if not line.startswith("#"):
            k, *v = line.split()
            gold[k] = [int(x) for x in v]
    r = binding.Router(cfg, wl.initial_state(cfg))
    out = r.route_step(wl.initial_waiting(cfg))
    assert out["assign"][0, :32].tolist() == gold["assign"] and out["best_g"][0, :32].tolist() == gold["best_g"]
    assert out["best_i"][0].tolist() == gold["best_i"] and out["stats"][0, :10].tolist() == gold["stats"]
    st = r.state()
    assert st["L"][0].tolist() == gold["L"] and st["n"][0].tolist() == gold["n"]
    r.advance(1)
    st = r.state()
    assert st["L"][0].tolist() == gold["L1"] and st["n"][0].tolist() == gold["n1"]
    r.close()


def test_brh_rounds_against_stored_values():
    """The HIP path against tests/golden/brh_rounds.txt (the oracle's stored results for a short- and a
    long-horizon round): assignments, reductions, statistics, loads, projection rows and score bit patterns."""
    import importlib.util
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_brh_golden", os.path.join(here, "make_brh_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    gold = {}
    for line in open(os.path.join(here, "brh_rounds.txt")):
        if not line.startswith("#"):
            k, *v = line.split()
            gold[k] = [int(x) for x in v]
    for tag, kw in mod.CASES:
        _say(f"stored BR-H round {tag}")
        cfg, init, arr = mod.case_inputs(kw)
        r = binding.Router(cfg, init)
        out = r.route_step(arr)
        st = r.state()
        assert out["assign"].ravel().tolist() == gold[f"{tag}.assign"]
        assert out["best_g"].ravel().tolist() == gold[f"{tag}.best_g"] and out["best_i"].ravel().tolist() == gold[f"{tag}.best_i"]
        assert out["stats"][:, :12].ravel().tolist() == gold[f"{tag}.stats"]
        assert st["L"].ravel().tolist() == gold[f"{tag}.L"] and st["n"].ravel().tolist() == gold[f"{tag}.n"]
        assert st["Lh"][0].ravel().tolist() == gold[f"{tag}.Lh0"]
        assert np.asarray(out["F"][0, 0], np.float32).view(np.int32).tolist() == gold[f"{tag}.F0bits"]
        r.advance(1)
        st = r.state()
        assert st["L"].ravel().tolist() == gold[f"{tag}.L1"] and st["n"].ravel().tolist() == gold[f"{tag}.n1"]
        r.close()


CASES = [
    # (G, B, Q, H, extra)                        spans every register layout (Q<=256/512/1024/2048)
    (4, 16, 32, 0, {}),
    (16, 24, 256, 0, {}),
    (16, 24, 200, 0, dict(tie_heavy=True)),
    (7, 9, 300, 0, dict(R_max=3)),
    (33, 40, 700, 0, dict(R_max=8, S_greedy=40)),
    (64, 12, 2048, 0, dict(R_max=5)),
    (1, 8, 64, 0, {}),
    (5, 1, 17, 0, dict(R_max=1)),
    (16, 20, 256, 0, dict(token_watermark=30000, token_cap=28000)),
    (8, 16, 128, 0, dict(S_greedy=0)),
    (8, 16, 128, 0, dict(S_greedy=10 ** 6)),
    (8, 16, 96, 4, dict(gate_pfin=0.0)),
    (8, 16, 96, 4, dict(gate_pfin=0.5)),
    (32, 24, 512, 4, dict(gate_pfin=0.0, gamma=0.64, beta=14.67)),
    (64, 10, 2048, 8, dict(gate_pfin=0.0, R_max=4)),
    (13, 30, 333, 8, dict(gate_pfin=0.3, R_max=8, tie_heavy=True)),
    (16, 20, 256, 3, dict(pred_mode=1)),
    (16, 20, 256, 8, dict(gate_pfin=0.0, token_watermark=40000)),
    (6, 12, 64, 1, dict(gate_pfin=0.0, gamma=1.0)),
    # horizons beyond 8: per-offset state in LDS (Sec. 6 deploys H = 80)
    (8, 16, 96, 80, dict(pred_mode=1, R_max=4, gamma=0.97)),
    (16, 20, 256, 9, dict(pred_mode=1)),
    (33, 12, 600, 128, dict(pred_mode=1, R_max=8, gamma=0.99)),
    (64, 10, 2048, 80, dict(pred_mode=1, R_max=4, gamma=0.95)),
    (13, 30, 333, 63, dict(pred_mode=1, tie_heavy=True, token_watermark=40000)),
    (6, 12, 1000, 64, dict(pred_mode=1, gamma=1.0, S_greedy=0)),
    # candidate windows of 9..16 requests (exhaustive search over up to 2^16 subsets per pop)
    (16, 24, 256, 0, dict(R_max=12)),
    (7, 12, 300, 0, dict(R_max=16, S_greedy=10 ** 6)),
    (33, 40, 700, 0, dict(R_max=9, S_greedy=40, tie_heavy=True)),
    (64, 20, 2048, 0, dict(R_max=10)),
    (8, 24, 96, 4, dict(gate_pfin=0.0, R_max=16)),
    (13, 30, 333, 8, dict(gate_pfin=0.3, R_max=11, tie_heavy=True)),
    (16, 20, 1000, 3, dict(pred_mode=1, R_max=13, token_watermark=40000)),
    (8, 16, 96, 80, dict(pred_mode=1, R_max=12, gamma=0.97)),
    (5, 8, 600, 9, dict(pred_mode=1, R_max=16, S_greedy=10 ** 6)),
    # candidate windows of 17..32 requests: the search by reachable sums (bit rows in LDS or in the workspace)
    (16, 24, 256, 0, dict(R_max=24)),
    (7, 12, 300, 0, dict(R_max=32, S_greedy=10 ** 6)),
    (33, 40, 700, 0, dict(R_max=20, S_greedy=40, tie_heavy=True)),
    (64, 20, 2048, 0, dict(R_max=17)),
    (8, 24, 96, 4, dict(gate_pfin=0.0, R_max=32)),
    (13, 30, 333, 8, dict(gate_pfin=0.3, R_max=27, tie_heavy=True)),
    (16, 20, 1000, 3, dict(pred_mode=1, R_max=19, token_watermark=40000)),
    (1, 40, 200, 0, dict(R_max=32, S_greedy=10 ** 6)),
    (3, 9, 128, 0, dict(R_max=32, S_greedy=10 ** 6, tie_heavy=True)),
    # the two stages (p_fin, mu_rem) supplied per request
    (16, 20, 256, 6, dict(pred_mode=3, gate_pfin=0.5)),
    (32, 100, 512, 4, dict(pred_mode=3, gate_pfin=0.0)),
    (8, 16, 96, 80, dict(pred_mode=3, gate_pfin=0.5, gamma=0.97)),
    # the largest LDS footprint: longest queue, longest horizon, widest window
    (3, 6, 2048, 128, dict(pred_mode=1, R_max=16, gamma=0.99)),
    # many equal lengths at long horizons: the bracketing search cannot separate equal scores and hands over to
    # the full scan (shared by the cluster's waves), for every queue size class
    (8, 24, 256, 40, dict(pred_mode=1, tie_heavy=True)),
    (5, 30, 512, 24, dict(pred_mode=1, tie_heavy=True, gamma=1.0)),
    (9, 20, 1024, 100, dict(pred_mode=3, tie_heavy=True, gate_pfin=0.0)),
    (4, 40, 2048, 16, dict(pred_mode=1, tie_heavy=True, token_watermark=30000)),
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_random_rounds(case):
    G, B, Q, H, extra = CASES[case]
    for seed in range(3):
        kw = dict(extra)
        _say(f"case {case} seed {seed}: G={G} B={B} Q={Q} H={H} {kw}")
        cfg, init, arr = wl.random_case(1000 * case + seed, N=6, G=G, B=B, max_wait=Q, H=H,
                                        fill=[0.3, 0.6, 0.9][seed], s_hi=[4096, 32768, 512][seed], **kw)
        oc, r = run_pair(cfg, init, arr, tag=f"case{case}/{seed}")
        # a second and third round on the evolved state, with fresh arrivals and ragged counts
        for rnd in range(2):
            _, _, arr2 = wl.random_case(77 + 1000 * case + seed + rnd, N=6, G=G, B=B, max_wait=Q, H=H,
                                        n_wait=max(1, Q // 3), **kw)
            ref = oc.route_step(arr2)
            out = r.route_step(arr2, advance=3 if rnd else 0)      # second one: round + decode steps in one launch
            compare_outputs(ref, out, cfg, f"case{case}/{seed}/r{rnd}")
            oc.advance(2 + rnd)
            if rnd == 0:
                r.advance(2)
            compare_state(oc, r.state(), cfg, f"case{case}/{seed}/r{rnd}")
        r.close()


@pytest.mark.parametrize("G,B,Q,H,extra", [
    (16, 24, 256, 0, {}),
    (7, 9, 200, 0, dict(token_watermark=30000, token_cap=28000, tie_heavy=True)),
    (64, 6, 70, 0, dict(R_max=5)),
    (3, 8, 512, 0, {}),
    (33, 12, 100, 4, dict(gate_pfin=0.0)),
    (12, 6, 300, 8, dict(pred_mode=1)),
    (12, 10, 130, 3, dict(gate_pfin=0.5, gamma=0.64, beta=14.67, tie_heavy=True)),
    (16, 12, 256, 0, dict(R_max=12)),                    # wide windows: reductions and round as separate launches
    (8, 10, 100, 40, dict(pred_mode=1, gamma=0.97)),     # long horizon: block-per-cluster score kernel; two waves share a cluster's searches
    (5, 8, 90, 24, dict(pred_mode=1, n_inst=2304)),      # long horizon, more clusters than share waves: one wave per cluster
    (6, 8, 300, 16, dict(pred_mode=1, n_inst=1200, gate_pfin=0.0)),  # queues of up to 512: two waves at this batch size
    # windows beyond 16 requests on batches too large for a block of four waves per cluster: one wave builds the rows
    (4, 6, 60, 0, dict(R_max=20, n_inst=1100, S_greedy=4)),
    (5, 7, 70, 4, dict(R_max=24, n_inst=1100, gate_pfin=0.0, S_greedy=5)),
])
def test_many_small_clusters(G, B, Q, H, extra):
    """Batches of 2048 clusters and more with short queues take the one-wave-per-cluster score kernel
    (no matrix requested): per-request best worker and per-worker best request against the oracle,
    with ragged queue lengths, full workers and the watermark filter."""
    extra = dict(extra)
    N = extra.pop("n_inst", 2048)
    _say(f"many small clusters N={N} G={G} B={B} Q={Q} H={H} {extra}")
    cfg, init, arr = wl.random_case(500 + G + Q + H, N=N, G=G, B=B, max_wait=Q, H=H, fill=0.8, **extra)
    oc, r = run_pair(cfg, init, arr, matrix=False, tag="small clusters")
    _, _, arr2 = wl.random_case(900 + G + Q + H, N=N, G=G, B=B, max_wait=Q, H=H, n_wait=max(1, Q // 5), **extra)
    compare_outputs(oc.route_step(arr2), r.route_step(arr2, matrix=False, advance=1), cfg, "small clusters r2")
    oc.advance(1)
    compare_state(oc, r.state(), cfg, "small clusters r2")
    r.close()


@pytest.mark.parametrize("G,B,Q,n0,lengths", [
    (16, 40, 256, 20, (50, 90)),        # ~6 requests per length: groups inside the 64 shortest
    (16, 40, 256, 20, (500, 503)),      # 3 lengths, ~85 each: groups wider than 64
    (16, 40, 256, 20, (16, 4000)),      # mostly distinct
    (64, 12, 700, 4, (100, 140)),       # 11 registers of keys per lane, wide level
    (5, 70, 512, 10, (30, 33)),
    (2, 200, 300, 50, (7, 9)),
])
def test_balanced_clusters_equal_lengths(G, B, Q, n0, lengths):
    """BR-0 clusters whose workers carry equal (or nearly equal) loads, so that no waiting request is
    below a margin and the shortest-request rule decides nearly every admission, with many requests of
    equal length (order of admission among equals: arrival order)."""
    N = 12
    rng = np.random.default_rng(G * 1000 + Q + lengths[0])
    cfg = wl.RouteConfig(name="balanced", n_inst=N, G=G, B=B, max_wait=Q, H=0)
    n = np.full((N, G), n0, np.int32)
    kv = np.zeros((N, G, B), np.int32)
    rem = np.zeros((N, G, B), np.int32)
    kv[:, :, :n0] = 1000
    kv[N // 2:, :, 0] += rng.integers(0, 3 * lengths[0], size=(N - N // 2, G)).astype(np.int32)  # second half: small spread
    rem[:, :, :n0] = rng.integers(1, 6, size=(N, G, n0))
    init = wl.InitState(n=n, kv=kv, rem=rem, pred=None)
    _say(f"balanced clusters G={G} B={B} Q={Q} lengths={lengths}")
    oc, r = br_oracle.OracleCluster(cfg, init), binding.Router(cfg, init)
    for rnd in range(4):
        cnt = rng.integers(Q // 2, Q + 1, size=N).astype(np.int32)
        s = rng.integers(lengths[0], lengths[1], size=(N, Q)).astype(np.int32)
        o = rng.integers(1, 5, size=(N, Q)).astype(np.int32)
        arr = wl.Arrivals(count=cnt, s=s, o=o, id=np.arange(N * Q, dtype=np.int32).reshape(N, Q) + rnd * N * Q, pred=None)
        ref = oc.route_step(arr)
        out = r.route_step(arr, advance=rnd % 2)
        compare_outputs(ref, out, cfg, f"balanced r{rnd}")
        oc.advance(1)
        if rnd % 2 == 0:
            r.advance(1)
        compare_state(oc, r.state(), cfg, f"balanced r{rnd}")
    r.close()


@pytest.mark.parametrize("seed", [11, 12])
def test_random_shapes_equal_lengths_and_loads(seed):
    """Many small BR-0 shapes drawn at random, built to produce ties: few distinct request lengths,
    equal or nearly equal worker loads, thresholds from "refined stage only" to "greedy stage only".
    This is where the admission shortcuts of the assignment kernel must still follow the one-by-one loop."""
    rng = np.random.default_rng(seed)
    for case in range(60):
        G = int(rng.choice([2, 3, 5, 8, 16, 16, 31, 64]))
        Q = int(rng.choice([64, 100, 256, 256, 300, 512, 700, 1024, 2048]))
        B = int(rng.integers(2, 60))
        N = int(rng.choice([7, 64, 300])) if Q < 1024 else 8
        R_max = int(rng.choice([1, 2, 4, 4, 4, 6, 8]))
        S_greedy = int(rng.choice([0, G, G * R_max, G * R_max, 3 * G * R_max, 10 ** 6]))
        n0 = int(rng.integers(0, B))
        spread = int(rng.choice([0, 0, 5, 50, 500, 5000, 50000]))
        lo = int(rng.choice([1, 5, 50, 500, 3000]))
        width = int(rng.choice([1, 2, 3, 10, 100, 1000, 20000]))
        # a token watermark around the loads in a third of the shapes: some workers can take nothing
        wm = int(rng.choice([0, 0, 0, 0, 1000 * n0 + lo, 1000 * n0 + 2 * (lo + width), 1000 * n0 + 6 * (lo + width)]))
        cfg = wl.RouteConfig(name="shapes", n_inst=N, G=G, B=B, max_wait=Q, H=0, R_max=R_max, S_greedy=S_greedy,
                             token_watermark=wm, token_cap=wm)
        n = np.full((N, G), n0, np.int32)
        n[:, ::3] = rng.integers(0, B + 1, size=n[:, ::3].shape)
        kv = np.zeros((N, G, B), np.int32)
        rem = np.zeros((N, G, B), np.int32)
        used = np.arange(B)[None, None, :] < n[:, :, None]
        kv[used] = 1000
        if spread:
            kv[:, :, 0] += rng.integers(0, spread + 1, size=(N, G)).astype(np.int32) * (n > 0)
        rem[used] = rng.integers(1, 4, size=int(used.sum()))
        init = wl.InitState(n=n, kv=kv, rem=rem, pred=None)
        tag = f"shapes {seed}/{case}: W={wm} N={N} G={G} B={B} Q={Q} R_max={R_max} S_greedy={S_greedy} n0={n0} spread={spread} s in [{lo},{lo + width})"
        _say(tag)
        oc, r = br_oracle.OracleCluster(cfg, init), binding.Router(cfg, init)
        for rnd in range(3):
            cnt = rng.integers(0, Q + 1, size=N).astype(np.int32)
            s = rng.integers(lo, lo + width, size=(N, Q)).astype(np.int32)
            o = rng.integers(1, 4, size=(N, Q)).astype(np.int32)
            arr = wl.Arrivals(count=cnt, s=s, o=o, id=np.arange(N * Q, dtype=np.int32).reshape(N, Q), pred=None)
            ref = oc.route_step(arr, want_scores=False)
            out = r.route_step(arr, scores=False, advance=rnd % 2)
            compare_outputs(ref, out, cfg, f"{tag} r{rnd}")
            oc.advance(1)
            if rnd % 2 == 0:
                r.advance(1)
            compare_state(oc, r.state(), cfg, f"{tag} r{rnd}")
        r.close()


@pytest.mark.parametrize("long_h", [False, True])
def test_random_shapes_horizon(long_h):
    """Many small BR-H shapes drawn at random: every prediction mode (hazards, direct estimate, estimate kept
    by the library with initial (estimate, age, phase) triples), gates, discounts, weights, thresholds.
    long_h: horizons 9..128 (direct or maintained estimate), the kernels that keep the offsets in LDS."""
    rng = np.random.default_rng(43 if long_h else 41)
    for case in range(30 if long_h else 50):
        G = int(rng.choice([2, 3, 8, 16, 31, 64]))
        Q = int(rng.choice([64, 100, 256, 300, 512, 700, 1024, 2048]))
        B = int(rng.integers(2, 50))
        N = int(rng.choice([3, 16, 64])) if Q < 1024 else 4
        H = int(rng.choice([9, 12, 16, 33, 64, 65, 80, 127, 128])) if long_h else int(rng.integers(1, 9))
        mode = int(rng.choice([1, 2, 3])) if long_h else int(rng.choice([0, 0, 1, 2, 3]))
        kw = dict(R_max=int(rng.choice([1, 2, 4, 4, 8])), gate_pfin=float(rng.choice([0.0, 0.3, 0.5])),
                  gamma=float(rng.choice([0.9, 0.97, 1.0] if long_h else [0.64, 0.9, 1.0])),
                  beta=float(rng.choice([-1.0, 14.67, 0.5, 2.0])),
                  tie_heavy=bool(rng.integers(0, 2)), s_hi=int(rng.choice([64, 4096, 32768])),
                  fill=float(rng.choice([0.2, 0.6, 0.95])))
        if mode == 2:
            kw["refresh_period"] = int(rng.integers(0, 5))
        if kw["beta"] < 0:
            kw.pop("beta")
        S_greedy = int(rng.choice([0, G, 4 * G, 10 ** 6]))
        cfg, init, arr = wl.random_case(int(rng.integers(1, 10 ** 6)), N=N, G=G, B=B, max_wait=Q, H=H, pred_mode=mode,
                                        S_greedy=S_greedy, **kw)
        hist = wl.output_history(cfg, 500) if mode == 2 else None
        tag = f"horizon shapes {case}: N={N} G={G} B={B} Q={Q} H={H} mode={mode} S_greedy={S_greedy} {kw}"
        _say(tag)
        oc, r = br_oracle.OracleCluster(cfg, init, hist=hist), binding.Router(cfg, init, hist=hist)
        for rnd in range(3):
            if rnd:
                _, _, arr = wl.random_case(int(rng.integers(1, 10 ** 6)), N=N, G=G, B=B, max_wait=Q, H=H, pred_mode=mode,
                                           n_wait=max(1, Q // 3), **{k: v for k, v in kw.items() if k != "fill"})
            ref = oc.route_step(arr, want_prep=True)
            out = r.route_step(arr, advance=rnd % 2)
            if rnd % 2 == 0:
                compare_prep(ref, r.state(), f"{tag} r{rnd}")
            compare_outputs(ref, out, cfg, f"{tag} r{rnd}")
            oc.advance(1)
            if rnd % 2 == 0:
                r.advance(1)
            compare_state(oc, r.state(), cfg, f"{tag} r{rnd}")
        r.close()


def test_edge_cases():
    # no arrivals at all (NULL), empty queue
    cfg, init, arr = wl.random_case(5, N=3, G=4, B=8, max_wait=32, H=0)
    _say("edge: null arrivals")
    oc, r = br_oracle.OracleCluster(cfg, init), binding.Router(cfg, init)
    ref, out = oc.route_step(None), r.route_step(None)
    compare_outputs(ref, out, cfg, "null")
    compare_state(oc, r.state(), cfg, "null")
    # zero counts
    arr0 = wl.Arrivals(np.zeros_like(arr.count), arr.s, arr.o, arr.id, arr.pred)
    compare_outputs(oc.route_step(arr0), r.route_step(arr0), cfg, "zero")
    # count beyond the queue cap -> drops; then nothing free -> everything deferred
    _say("edge: overflow")
    arrx = wl.Arrivals(np.full_like(arr.count, arr.s.shape[1]), arr.s, arr.o, arr.id, arr.pred)
    for k in range(3):
        compare_outputs(oc.route_step(arrx), r.route_step(arrx), cfg, f"overflow{k}")
        compare_state(oc, r.state(), cfg, f"overflow{k}")
    r.close()
    # all workers full: S_tot = 0
    _say("edge: full")
    cfg, init, arr = wl.random_case(6, N=2, G=4, B=8, max_wait=32, H=2, fill=1.0, gate_pfin=0.0)
    oc, r = run_pair(cfg, init, arr, tag="full")
    r.close()
    # empty cluster, more requests than slots
    _say("edge: empty cluster")
    cfg, init, arr = wl.random_case(8, N=2, G=3, B=4, max_wait=64, H=0, fill=0.0, n_wait=64)
    oc, r = run_pair(cfg, init, arr, tag="emptycluster")
    r.close()
    # maximum sizes
    _say("edge: max sizes")
    cfg, init, arr = wl.random_case(9, N=2, G=64, B=1024, max_wait=2048, H=8, fill=0.97, n_wait=2048,
                                    gate_pfin=0.0, R_max=8, s_hi=32768)
    oc, r = run_pair(cfg, init, arr, matrix=True, tag="max")
    r.close()


def test_edge_cases_long_horizon_and_wide_window():
    """The same degenerate inputs through the kernels for horizons beyond 8 and windows beyond 8 requests."""
    for tag, kw in (("H=80", dict(H=80, pred_mode=1)), ("H=128 pair", dict(H=128, pred_mode=3, gate_pfin=0.5)),
                    ("R_max=16", dict(H=0, R_max=16)), ("H=33 R_max=12", dict(H=33, pred_mode=1, R_max=12))):
        _say(f"edge long/wide: {tag}")
        cfg, init, arr = wl.random_case(15, N=3, G=4, B=8, max_wait=32, **kw)
        oc, r = br_oracle.OracleCluster(cfg, init), binding.Router(cfg, init)
        compare_outputs(oc.route_step(None), r.route_step(None), cfg, f"{tag} null")       # no arrivals at all
        compare_state(oc, r.state(), cfg, f"{tag} null")
        arrx = wl.Arrivals(np.full_like(arr.count, arr.s.shape[1]), arr.s, arr.o, arr.id, arr.pred)
        for k in range(3):                                                                 # overflow, then nothing free
            compare_outputs(oc.route_step(arrx), r.route_step(arrx, advance=k % 2), cfg, f"{tag} overflow{k}")
            if k % 2:
                oc.advance(1)
            compare_state(oc, r.state(), cfg, f"{tag} overflow{k}")
        r.close()
        cfg, init, arr = wl.random_case(16, N=2, G=4, B=8, max_wait=32, fill=1.0, **kw)    # all workers full
        oc, r = run_pair(cfg, init, arr, tag=f"{tag} full")
        r.close()
        cfg, init, arr = wl.random_case(18, N=2, G=3, B=4, max_wait=64, fill=0.0, n_wait=64, **kw)   # empty cluster
        oc, r = run_pair(cfg, init, arr, tag=f"{tag} empty")
        r.close()
        cfg, init, arr = wl.random_case(19, N=2, G=1, B=3, max_wait=5, fill=0.4, n_wait=5, **kw)     # one worker
        oc, r = run_pair(cfg, init, arr, tag=f"{tag} G=1")
        r.close()


def test_loads_at_the_edge_of_the_key_range():
    """Per-worker loads just below 2^25 (the range the library states: its worker keys pack a load into 25 bits):
    full parity and a zero range counter; and a one-worker cluster beyond it, where no ordering is involved:
    the counter reports it on both sides."""
    G, B, Q = 4, 1024, 256
    rng = np.random.default_rng(77)
    cfg = wl.RouteConfig(name="edge25", n_inst=3, G=G, B=B, max_wait=Q, H=0)
    n = np.array([[1020, 1019, 1021, 1018], [1023, 1023, 1022, 1023], [1000, 1016, 1016, 1010]], np.int32)
    kv = np.zeros((3, G, B), np.int32)
    rem = np.zeros((3, G, B), np.int32)
    used = np.arange(B)[None, None, :] < n[:, :, None]
    kv[used] = 32768
    rem[used] = rng.integers(2, 9, size=int(used.sum()))
    init = wl.InitState(n=n, kv=kv, rem=rem, pred=None)
    _say("loads just below 2^25")
    oc, r = br_oracle.OracleCluster(cfg, init), binding.Router(cfg, init)
    for rnd in range(3):
        s = rng.integers(20000, 30001, size=(3, Q)).astype(np.int32)
        arr = wl.Arrivals(count=np.array([40, 7, 256], np.int32), s=s, o=rng.integers(1, 5, size=(3, Q)).astype(np.int32),
                          id=np.arange(3 * Q, dtype=np.int32).reshape(3, Q), pred=None)
        ref, out = oc.route_step(arr), r.route_step(arr)
        compare_outputs(ref, out, cfg, f"edge25 r{rnd}")
        assert (ref["stats"][:, br_oracle.ST["load_range"]] == 0).all() and ref["stats"][:, br_oracle.ST["spread"]].max() < 1 << 25
        if rnd == 0:
            assert oc.L.max() > (1 << 25) - (1 << 21)      # the case does sit at the edge (later rounds: requests have left)
        oc.advance(1), r.advance(1)
        compare_state(oc, r.state(), cfg, f"edge25 r{rnd}")
    r.close()
    _say("one worker beyond 2^25")
    cfg = wl.RouteConfig(name="edge25b", n_inst=2, G=1, B=B, max_wait=16, H=0)
    n = np.array([[1000], [10]], np.int32)
    kv = np.zeros((2, 1, B), np.int32)
    rem = np.zeros((2, 1, B), np.int32)
    kv[0, 0, :1000], rem[0, 0, :1000] = 40000, 3
    kv[1, 0, :10], rem[1, 0, :10] = 500, 3
    init = wl.InitState(n=n, kv=kv, rem=rem, pred=None)
    oc, r = br_oracle.OracleCluster(cfg, init), binding.Router(cfg, init)
    arr = wl.Arrivals(count=np.array([5, 5], np.int32), s=np.full((2, 16), 100, np.int32), o=np.full((2, 16), 2, np.int32),
                      id=np.arange(32, dtype=np.int32).reshape(2, 16), pred=None)
    ref, out = oc.route_step(arr), r.route_step(arr)
    compare_outputs(ref, out, cfg, "edge25b")
    assert ref["stats"][:, br_oracle.ST["load_range"]].tolist() == [1, 0]
    ref, out = oc.route_bypass(arr), r.route_bypass(arr)
    assert np.array_equal(out["stats"], ref["stats"]) and ref["stats"][:, br_oracle.ST["load_range"]].tolist() == [1, 0]
    compare_state(oc, r.state(), cfg, "edge25b")
    r.close()


def test_advance_many_steps_closed_form():
    """n decode steps in one call equal n single steps of the oracle (requests leave mid-way)."""
    for H in (0, 4):
        cfg, init, arr = wl.random_case(21 + H, N=5, G=9, B=150, max_wait=64, H=H, fill=0.8, gate_pfin=0.0)
        _say(f"advance H={H}")
        oc, r = br_oracle.OracleCluster(cfg, init), binding.Router(cfg, init)
        for t in (1, 3, 7, 40):
            oc.advance(t)
            r.advance(t)
            compare_state(oc, r.state(), cfg, f"adv{t}")
        r.close()


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("name,steps,over", [
    ("c2", 400, dict()),
    ("c2", 300, dict(arrival_rate=4.0, seed=1001)),                    # balanced: stages alternate
    ("c3", 300, dict(gate_pfin=0.0)),
    ("c3", 200, dict(gate_pfin=0.5, beta=14.67, gamma=0.64)),
    ("c5", 150, dict(gate_pfin=0.0)),
])
def test_replay(name, steps, over, fused):
    """fused: br_route_advance (round + decode step in one launch) instead of the two calls."""
    cfg = wl.config(name, **over)
    _say(f"replay {name} {steps} {over} fused={fused}")
    tr = wl.arrival_trace(cfg, steps, informative=(name == "c3" and over.get("gate_pfin") == 0.5))
    oc, r = br_oracle.OracleCluster(cfg), binding.Router(cfg)
    for k in range(steps):
        a = tr.step(k)
        ref = oc.route_step(a, want_scores=(k % 25 == 0))
        out = r.route_step(a, scores=(k % 25 == 0), advance=int(fused))
        compare_outputs(ref, out, cfg, f"{name} step {k}")
        oc.advance(1)
        if not fused:
            r.advance(1)
        if k % 25 == 0 or k == steps - 1:
            compare_state(oc, r.state(), cfg, f"{name} step {k}")
    r.close()


def test_batched_replay_fused_steps():
    """bench.py's replay leg at reduced size: 48 instances of the BR-0 replay shape with their own arrival
    streams, 160 decode steps from empty, one fused call per step and nothing read back in between."""
    cfg = wl.config("c2", n_inst=48)
    steps = 160
    _say(f"batched replay {cfg.n_inst} x {steps}")
    tr = wl.arrival_trace(cfg, steps)
    oc, r = br_oracle.OracleCluster(cfg), binding.Router(cfg)
    out = r.alloc_outputs(scores=False)
    refs = []
    for k in range(steps):
        a = tr.step(k)
        r.route_advance_device(binding.DeviceArrivals(a, r.device, r.Pq), out, 1)
        ref = oc.route_step(a, want_scores=False)
        oc.advance(1)
        if k % 40 == 39 or k == steps - 1:
            r.stream.synchronize()
            got = {kk: out[kk].cpu().numpy() for kk in ("assign", "assign_id", "stats")}
            compare_outputs(ref, got, cfg, f"batched replay step {k}")
            compare_state(oc, r.state(), cfg, f"batched replay step {k}")
    r.close()


@pytest.mark.parametrize("fused", [False, True])
def test_c4_full_size_bench_configuration(fused):
    """The batched throughput workload at full size, in the launch configurations bench.py times
    (no score matrix written, best_g / best_i on; round and decode step as two calls or as the one
    fused call): every instance against the oracle."""
    cfg = wl.config("c4")
    _say(f"c4 full size fused={fused}")
    init, arr = wl.initial_state(cfg), wl.initial_waiting(cfg)
    oc, r = br_oracle.OracleCluster(cfg, init), binding.Router(cfg, init)
    ref = oc.route_step(arr)
    out = r.route_step(arr, matrix=False, advance=int(fused))
    compare_outputs(ref, out, cfg, "c4")
    assert (ref["stats"][:, br_oracle.ST["admitted"]] == 256).all()
    oc.advance(1)
    if not fused:
        r.advance(1)
    compare_state(oc, r.state(), cfg, "c4")
    r.close()


@pytest.mark.parametrize("name,over", [("c2", {}), ("c3", dict(gate_pfin=0.5)), ("c5", {})])
def test_replay_full_length(name, over):
    """The replay workloads at their full length (2000 / 1000 / 10000 decode steps): assignments and
    statistics of every step, the whole state every 250 steps."""
    cfg = wl.config(name, **over)
    _say(f"full replay {name} {cfg.steps} steps")
    tr = wl.arrival_trace(cfg)
    oc, r = br_oracle.OracleCluster(cfg), binding.Router(cfg)
    out = r.alloc_outputs(scores=False)
    for k in range(cfg.steps):
        a = tr.step(k)
        ref = oc.route_step(a, want_scores=False)
        darr = binding.DeviceArrivals(a, r.device, r.Pq)
        r.route_step_device(darr, out)
        r.advance(1)
        r.stream.synchronize()
        got = {kk: out[kk].cpu().numpy() for kk in ("assign", "assign_id", "stats")}
        compare_outputs(ref, got, cfg, f"{name} step {k}")
        oc.advance(1)
        if k % 250 == 0 or k == cfg.steps - 1:
            compare_state(oc, r.state(), cfg, f"{name} step {k}")
        if k % 1000 == 0:
            _say(f"  step {k}")
    r.close()


@pytest.mark.parametrize("gate", [None, 0.0])
def test_brh_batched_bench_configuration(gate):
    """The batched BR-H side workload of bench.py at full size (4096 clusters), every instance; also with
    the p_fin gate off (then no request counts at the last offset and every score is negative)."""
    over = {} if gate is None else dict(gate_pfin=gate)
    cfg = wl.config("c3", n_inst=4096, token_watermark=0, **over, token_cap=0, init_active_per_worker=76,
                    init_kv_lo=256, init_kv_hi=8192, init_rem_lo=1, init_rem_hi=1024, init_waiting=256)
    _say("brh batched full size")
    init, arr = wl.initial_state(cfg), wl.initial_waiting(cfg)
    oc, r = br_oracle.OracleCluster(cfg, init), binding.Router(cfg, init)
    ref = oc.route_step(arr, want_prep=True)
    out = r.route_step(arr, matrix=False)
    from tests.parity import compare_prep
    compare_prep(ref, r.state(), "brh batch")
    compare_outputs(ref, out, cfg, "brh batch")
    assert (ref["stats"][:, br_oracle.ST["admitted"]] > 0).all()
    oc.advance(1)
    r.advance(1)
    compare_state(oc, r.state(), cfg, "brh batch")
    r.close()


def test_long_horizon_batched_bench_configuration():
    """bench.py's batched leg at the paper's horizon and window (2048 clusters, H=80, G=8, R_max=4, estimate
    maintained by the library) through the fused entry point: every instance."""
    cfg = wl.config("c3", n_inst=2048, G=8, B=64, max_wait=256, H=80, R_max=4, pred_mode=2, token_watermark=0,
                    token_cap=0, init_active_per_worker=48, init_kv_lo=256, init_kv_hi=8192, init_rem_lo=1,
                    init_rem_hi=1024, init_waiting=256, seed=2100)
    _say("H=80 batched full size")
    hist = wl.output_history(cfg, 8000)
    init, arr = wl.initial_state(cfg), wl.initial_waiting(cfg)
    oc, r = br_oracle.OracleCluster(cfg, init, hist=hist), binding.Router(cfg, init, hist=hist)
    ref = oc.route_step(arr, want_prep=True)
    out = r.route_step(arr, matrix=False, advance=1)
    from tests.parity import compare_prep
    compare_prep(ref, r.state(), "h80 batch")
    compare_outputs(ref, out, cfg, "h80 batch")
    assert (ref["stats"][:, br_oracle.ST["admitted"]] == 128).all()
    oc.advance(1)
    compare_state(oc, r.state(), cfg, "h80 batch")
    r.close()


@pytest.mark.parametrize("R_max,S_greedy", [(16, 64), (32, 64), (32, 512)])
def test_wide_window_bench_configuration(R_max, S_greedy):
    """bench.py's wide-window legs at full size (1024 clusters of the c4 shape; R_max=16: every subset mask;
    R_max=32: reachable sums, with the main workload's threshold and with every admission in Stage 2) through
    the fused entry point; the oracle is slow on these, so it checks 200 sampled clusters one by one (clusters are
    independent), assignments, statistics and state."""
    import dataclasses
    cfg = wl.config("c4", n_inst=1024, R_max=R_max, S_greedy=S_greedy)
    _say(f"wide window full size R_max={R_max} S_greedy={S_greedy}")
    init, arr = wl.initial_state(cfg), wl.initial_waiting(cfg)
    r = binding.Router(cfg, init)
    out = r.route_step(arr, scores=False, advance=1)
    st = r.state()
    r.close()
    pick = np.random.default_rng(5).choice(cfg.n_inst, 200 if R_max == 16 else 60, replace=False)
    take = lambda obj: type(obj)(**{f.name: (None if getattr(obj, f.name) is None else getattr(obj, f.name)[pick])
                                    for f in dataclasses.fields(obj)})
    sub = dataclasses.replace(cfg, n_inst=len(pick))
    oc = br_oracle.OracleCluster(sub, take(init))
    ref = oc.route_step(take(arr), want_scores=False)
    got = {k: out[k][pick] for k in ("assign", "assign_id", "stats")}
    compare_outputs(ref, got, sub, "wide window")
    assert (ref["stats"][:, br_oracle.ST["stage2_pops"]] > 8).all()
    oc.advance(1)
    compare_state(oc, {k: (v[pick] if isinstance(v, np.ndarray) and v.shape[:1] == (cfg.n_inst,) else v) for k, v in st.items()},
                  sub, "wide window")


def test_wide_window_long_requests_reach_the_row_bound():
    """Windows of 32 requests with lengths up to 32768 and room for many per pop: subset sums beyond the length of
    the bit rows (131071) exist and are not candidates on either side; rows too long for LDS go to the workspace."""
    for seed, (G, B, H, fill, kw) in enumerate([(3, 12, 0, 0.3, {}), (2, 30, 0, 0.1, {}), (4, 10, 2, 0.3, dict(gate_pfin=0.0))]):
        _say(f"wide window, long requests: G={G} B={B} H={H}")
        cfg, init, arr = wl.random_case(700 + seed, N=3, G=G, B=B, max_wait=96, H=H, fill=fill, s_hi=32768, n_wait=96,
                                        R_max=32, S_greedy=10 ** 6, **kw)
        oc, r = run_pair(cfg, init, arr, tag=f"rowbound {seed}")
        r.close()


def test_pool_bypass():
    """br_route_bypass against the oracle: placements, loads, slot tables, queue fallback, drops."""
    for seed, (G, B, Q, cap, fill, wm) in enumerate([(4, 8, 16, 40, 0.5, 0), (16, 144, 256, 256, 0.85, 0),
                                                      (64, 12, 64, 900, 0.3, 0), (1, 5, 8, 20, 0.2, 0),
                                                      (16, 20, 32, 128, 0.6, 30000), (7, 9, 300, 2048, 0.1, 0)]):
        _say(f"bypass G={G} B={B} Q={Q} arrivals<={cap}")
        cfg, init, _ = wl.random_case(100 + seed, N=5, G=G, B=B, max_wait=Q, H=0, fill=fill, token_watermark=wm)
        _, _, arr = wl.random_case(200 + seed, N=5, G=G, B=B, max_wait=cap, H=0, s_hi=[4096, 16384, 32768][seed % 3])
        oc, r = br_oracle.OracleCluster(cfg, init), binding.Router(cfg, init)
        for rnd in range(2):
            ref, out = oc.route_bypass(arr), r.route_bypass(arr)
            for i in range(cfg.n_inst):
                c = int(arr.count[i])
                assert np.array_equal(out["assign"][i, :c], ref["assign"][i, :c]), (seed, rnd, i)
            assert np.array_equal(out["stats"], ref["stats"]), (seed, rnd, out["stats"][:2], ref["stats"][:2])
            compare_state(oc, r.state(), cfg, f"bypass {seed}/{rnd}")
            oc.advance(3)
            r.advance(3)
        # what was queued is served by an ordinary round afterwards
        ref, out = oc.route_step(None), r.route_step(None)
        compare_outputs(ref, out, cfg, f"bypass {seed} then round")
        compare_state(oc, r.state(), cfg, f"bypass {seed} then round")
        r.close()


@pytest.mark.parametrize("H,refresh,gate", [(4, 0, 0.0), (8, 3, 0.5), (8, 1, 0.0), (80, 0, 0.5), (24, 5, 0.0)])
def test_maintained_estimate_replay(H, refresh, gate):
    """pred_mode 2: c_hat kept by the library (empirical-survival estimator, periodic refresh, decrement,
    floor): replay with short outputs so that the estimate moves; slot tables incl. (c_hat, age, since)."""
    cfg = wl.config("c3", G=8, B=24, max_wait=128, H=H, pred_mode=2, refresh_period=refresh, gate_pfin=gate,
                    token_watermark=0, arrival_rate=14.0, out_mu=float(np.log(3.0 * H)), out_sigma=0.9, out_hi=400,
                    seed=70 + H + refresh)
    hist = wl.output_history(cfg, 3000)
    _say(f"maintained estimate H={H} refresh={cfg.refresh_eff} gate={gate}")
    steps = 300
    tr = wl.arrival_trace(cfg, steps)
    oc, r = br_oracle.OracleCluster(cfg, hist=hist), binding.Router(cfg, hist=hist)
    for k in range(steps):
        a = tr.step(k)
        ref = oc.route_step(a, want_scores=(k % 20 == 0), want_prep=True)
        out = r.route_step(a, scores=(k % 20 == 0))
        if k % 10 == 0:
            compare_prep(ref, r.state(), f"mode2 step {k}")
        compare_outputs(ref, out, cfg, f"mode2 step {k}")
        t = 1 if k % 7 else 3
        oc.advance(t)
        r.advance(t)
        if k % 10 == 0 or k == steps - 1:
            compare_state(oc, r.state(), cfg, f"mode2 step {k}")
        if k % 3 == 0:                                   # an extra round through the fused entry, no arrivals
            ref = oc.route_step(None, want_scores=False)
            out = r.route_step(None, scores=False, advance=2)
            compare_outputs(ref, out, cfg, f"mode2 fused {k}")
            oc.advance(2)
            if k % 30 == 0:
                compare_state(oc, r.state(), cfg, f"mode2 fused {k}")
    assert (oc.pred[..., 0][np.arange(cfg.B)[None, None, :] < oc.n[:, :, None]] < H).any()   # estimates did move
    r.close()


@pytest.mark.parametrize("name,over", [("c2", dict(arrival_rate=12.0)), ("c3", dict(gate_pfin=0.5)),
                                       ("c3", dict(H=80, pred_mode=3, G=8, max_wait=256, arrival_rate=10.0))])
def test_graph_capture_and_replay(name, over):
    """The entry points only enqueue kernels (no allocation, no synchronisation, no memset): one step of the
    serving loop (br_route_advance) is captured into a graph once and replayed for 40 steps, the arrivals of
    each step copied into the captured buffers beforehand (eager work between the replays); every replay is
    checked against the oracle, the whole state every tenth."""
    import torch
    cfg = wl.config(name, **over)
    steps = 40
    _say(f"graph replay {name} {over}")
    tr = wl.arrival_trace(cfg, steps)
    torch.cuda.synchronize()
    oc, r = br_oracle.OracleCluster(cfg), binding.Router(cfg, stream=torch.cuda.Stream())   # capture needs a stream of its own
    darr = binding.DeviceArrivals(tr.step(0), r.device, r.Pq)     # the buffers the graph reads
    out = r.alloc_outputs(scores=True, matrix=False)
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=r.stream):
        r.route_advance_device(darr, out, 1)
    # capture only records: the state is still the initial one
    for k in range(steps):
        a = tr.step(k)
        nxt = binding.DeviceArrivals(a, r.device, r.Pq)
        with torch.cuda.stream(r.stream):
            darr.count.copy_(nxt.count), darr.s.copy_(nxt.s), darr.o.copy_(nxt.o), darr.id.copy_(nxt.id)
            if darr.pred is not None:
                darr.pred.copy_(nxt.pred)
            graph.replay()
        r.stream.synchronize()
        ref = oc.route_step(a, want_scores=True)
        oc.advance(1)
        got = {kk: out[kk].cpu().numpy() for kk in ("assign", "assign_id", "stats", "best_g", "best_i")}
        compare_outputs({kk: ref[kk] for kk in got}, got, cfg, f"graph {name} step {k}")
        if k % 10 == 9:
            compare_state(oc, r.state(), cfg, f"graph {name} step {k}")
    r.close()


def test_determinism():
    cfg, init, arr = wl.random_case(31, N=16, G=16, B=24, max_wait=256, H=4, gate_pfin=0.0, tie_heavy=True)
    outs = []
    for _ in range(2):
        r = binding.Router(cfg, init)
        outs.append(r.route_step(arr))
        r.close()
    for k in outs[0]:
        assert np.array_equal(outs[0][k], outs[1][k]), k
