"""Pins for the oracle's routing round, decode step and horizon projection.

The checks use only what the paper fixes (Sec. 2.2 load model, Sec. 3.1 objective,
Alg. BR-0 / BR-H structure) computed independently in Python, hand-worked examples,
and brute force on tiny instances.
"""
import itertools

import numpy as np
import pytest

from paper_2605_06113_amd import workloads as wl


def _mk(orc, cfg, init=None, **kw):
    return orc.OracleCluster(cfg, init, **kw)  # kw: force_float, hist


def _arr(s, o=None, ids=None, pred=None):
    s = np.asarray(s, np.int32)[None, :]
    n = s.shape[1]
    o = np.full((1, n), 5, np.int32) if o is None else np.asarray(o, np.int32)[None, :]
    ids = np.arange(n, dtype=np.int32)[None, :] if ids is None else np.asarray(ids, np.int32)[None, :]
    return wl.Arrivals(np.array([n], np.int32), s, o, ids, pred)


def _init(n, kv_rows, B, rem=50):
    G = len(n)
    st = wl.InitState(np.array([n], np.int32), np.zeros((1, G, B), np.int32),
                      np.zeros((1, G, B), np.int32), None)
    for g, row in enumerate(kv_rows):
        st.kv[0, g, :len(row)] = row
        st.rem[0, g, :len(row)] = rem
    return st


# ---- hand-worked rounds (Alg. BR-0) ----------------------------------------------------

def test_hand_worked_stage1(orc):
    # G=2, one free slot each, loads (100, 40); waiting 50, 30, 20; Stage 1 only (S_greedy = 0).
    # Step 1: caps tie -> lighter worker 1 (margin 60): scores 50,30,20 -> takes 50; loads (100, 90).
    # Step 2: worker 0 (margin 0): scores -30 (30), -20 (20) -> takes 20; loads (120, 90).
    cfg = wl.RouteConfig(name="h1", n_inst=1, G=2, B=2, max_wait=8, R_max=2, S_greedy=0)
    oc = _mk(orc, cfg, _init([1, 1], [[100], [40]], 2))
    out = oc.route_step(_arr([50, 30, 20]), want_events=True)
    assert out["assign"][0, :3].tolist() == [1, -1, 0]
    assert oc.L[0].tolist() == [120, 90]
    ev = out["events"][0][:out["n_events"][0]]
    assert [(e["g"], e["delta"], e["score"], e["stage"]) for e in ev] == [(1, 50, 50.0, 1), (0, 20, -20.0, 1)]
    st = out["stats"][0]
    assert st[orc.ST["admitted"]] == 2 and st[orc.ST["deferred"]] == 1 and st[orc.ST["stage1"]] == 2
    assert st[orc.ST["I_before"]] == 2 * 100 - 140 and st[orc.ST["I_after"]] == 2 * 120 - 210
    assert oc.qlen[0] == 1 and oc.qs[0, 0] == 30


def test_hand_worked_stage2(orc):
    # G=2, B=4, R_max=2, Stage 2 only.  loads (100, 40), caps (1, 2); waiting 50, 30, 20.
    # pop 1 (cap 2, margin 60): window {50,30}: F(50)=50, F(30)=30, F(80)=80-2*20=40 -> {50}.
    # loads (100, 90), caps (1, 1): margins (0, 10) -> pop 1: window {30,20}: F(30)=30-2*20=-10,
    #   F(20)=20-2*10=0, pair exceeds cap -> best 0 is not positive -> guard -> single best = 20 (F=0).
    # loads (100, 110): pop 0 (margin 10): window {30}: F=30-2*20=-10 -> guard -> 30.
    cfg = wl.RouteConfig(name="h2", n_inst=1, G=2, B=4, max_wait=8, R_max=2, S_greedy=100)
    oc = _mk(orc, cfg, _init([3, 2], [[60, 30, 10], [25, 15]], 4))
    out = oc.route_step(_arr([50, 30, 20]), want_events=True)
    assert out["assign"][0, :3].tolist() == [1, 0, 1]
    assert oc.L[0].tolist() == [130, 110]
    ev = out["events"][0][:out["n_events"][0]]
    assert [(e["g"], e["delta"], e["score"], e["stage"]) for e in ev] == \
        [(1, 50, 50.0, 2), (1, 20, 0.0, 3), (0, 30, -10.0, 3)]
    st = out["stats"][0]
    assert st[orc.ST["stage2_pops"]] == 3 and st[orc.ST["guard"]] == 2 and st[orc.ST["stage1"]] == 0
    assert oc.qlen[0] == 0


def test_hand_worked_subset_pair_wins(orc):
    # margin 100 on the only free worker: window {70, 30, 20}: the pair 70+30 fills the margin exactly.
    cfg = wl.RouteConfig(name="h3", n_inst=1, G=2, B=4, max_wait=8, R_max=3, S_greedy=100)
    oc = _mk(orc, cfg, _init([4, 1], [[50, 50, 50, 50], [100]], 4))
    out = oc.route_step(_arr([70, 30, 20]), want_events=True)
    e = out["events"][0][0]
    assert (e["g"], e["delta"], e["score"], e["n_req"]) == (1, 100, 100.0, 2)
    # afterwards margin 0, cap 1: best remaining single 20 scores -20 -> guard admits it
    assert out["assign"][0, :3].tolist() == [1, 1, 1]


def test_snapshot_scores_and_reductions(orc):
    cfg = wl.RouteConfig(name="h4", n_inst=1, G=3, B=2, max_wait=8)
    oc = _mk(orc, cfg, _init([1, 2, 0], [[100], [30, 30], []], 2))
    out = oc.route_step(_arr([50, 40, 120]))
    # M = 100, margins (0, 40, 100); worker 1 is full
    F = out["F"][0, :3]
    assert F.tolist() == [[50 - 3 * 50, 50 - 3 * 10, 50], [40 - 3 * 40, 40, 40], [120 - 3 * 120, 120 - 3 * 80, 120 - 3 * 20]]
    assert out["best_g"][0, :3].tolist() == [2, 2, 2]          # worker 1 has no free slot
    assert out["best_i"][0].tolist() == [1, -1, 2]             # w0: max(-100,-80,-240); w2: max(50,40,60)


def test_snapshot_reductions_tie_rules_hand_worked(orc):
    # Equal snapshot scores.  Per request: the lowest worker index.  Per worker: the longer request, then the
    # earlier arrival (the rule of argmax_i F_g({i}) in the round: lowest position in the order "longest first,
    # arrival order among equals").
    # G=3, loads (40, 40, 100): M = 100, margins (60, 60, 0), one free slot each.
    cfg = wl.RouteConfig(name="h5", n_inst=1, G=3, B=2, max_wait=8)
    oc = _mk(orc, cfg, _init([1, 1, 1], [[40], [40], [100]], 2))
    # waiting 40, 70, 40, 50: on workers 0 and 1 (margin 60): F(40) = 40, F(70) = 70 - 3*10 = 40, F(50) = 50;
    # on worker 2 (margin 0): F(s) = -2 s: -80, -140, -80, -100
    out = oc.route_step(_arr([40, 70, 40, 50]))
    assert out["F"][0, :4].tolist() == [[40, 40, -80], [40, 40, -140], [40, 40, -80], [50, 50, -100]]
    assert out["best_g"][0, :4].tolist() == [0, 0, 0, 0]        # workers 0 and 1 tie on every request: lowest index
    assert out["best_i"][0].tolist() == [3, 3, 0]               # worker 2: -80 twice: equal lengths, earlier arrival
    # without the 50: three requests tie at 40 on workers 0 and 1: the longer one (70, position 1) wins
    oc = _mk(orc, cfg, _init([1, 1, 1], [[40], [40], [100]], 2))
    out = oc.route_step(_arr([40, 70, 40]))
    assert out["best_i"][0].tolist() == [1, 1, 0]
    # a full worker is no candidate: ties then resolve among the rest
    oc = _mk(orc, cfg, _init([2, 1, 1], [[20, 20], [40], [100]], 2))
    out = oc.route_step(_arr([40, 70, 40]))
    assert out["best_g"][0, :3].tolist() == [1, 1, 1] and out["best_i"][0].tolist() == [-1, 1, 0]


# ---- structural invariants over replays -----------------------------------------------

def _replay_cfg(H, **kw):
    base = dict(name="mini", n_inst=1, G=4, B=8, max_wait=24, H=H, R_max=3, arrival_rate=3.0,
                prompt_mu=float(np.log(300.0)), prompt_hi=4096, out_mu=float(np.log(12.0)), out_sigma=0.8,
                out_hi=200, seed=5 + H, gate_pfin=0.0, gamma=0.8)
    base.update(kw)
    return wl.RouteConfig(**base)


@pytest.mark.parametrize("H", [0, 3])
@pytest.mark.parametrize("rate", [1.0, 3.0, 9.0])
def test_replay_matches_definition_of_load(orc, H, rate):
    """Per-worker loads equal sum over active requests of (s_i + k - x_i) (Sec. 2.2), with
    assignments sticky and every request served for exactly o_i steps."""
    cfg = _replay_cfg(H, arrival_rate=rate)
    steps = 250
    tr = wl.arrival_trace(cfg, steps, informative=True)
    oc = _mk(orc, cfg)
    placed = {}                  # id -> (g, s, o, x)
    info = {}
    for k in range(steps):
        a = tr.step(k)
        for j in range(int(a.count[0])):
            info[int(a.id[0, j])] = (int(a.s[0, j]), int(a.o[0, j]))
        S_tot = int((cfg.B - oc.n[0]).sum())
        out = oc.route_step(a, want_events=True)
        st = out["stats"][0]
        qn = int(st[orc.ST["qlen"]])
        # every queue entry decided at most once; bound ids never seen before (disjointness)
        for j in range(qn):
            g = int(out["assign"][0, j])
            rid = int(out["assign_id"][0, j])
            if g >= 0:
                assert rid not in placed
                s, o = info[rid]
                placed[rid] = (g, s, o, k)
        # work conservation (token filter off): every free slot is used while requests wait
        assert st[orc.ST["admitted"]] == min(S_tot, qn)
        assert st[orc.ST["deferred"]] == qn - st[orc.ST["admitted"]] == oc.qlen[0]
        # loads by the definition, at step k
        L = np.zeros(cfg.G, np.int64)
        cnt = np.zeros(cfg.G, np.int64)
        for rid, (g, s, o, x) in placed.items():
            if x <= k < x + o:
                L[g] += s + (k - x)
                cnt[g] += 1
        assert oc.L[0].tolist() == L.tolist()
        assert oc.n[0].tolist() == cnt.tolist() and (cnt <= cfg.B).all()
        for g in range(cfg.G):
            assert oc.kv[0, g, :oc.n[0, g]].sum() == L[g]
        assert st[orc.ST["I_after"]] == cfg.G * L.max() - L.sum()
        assert st[orc.ST["spread"]] == L.max() - L.min()
        if H == 0:   # telescoping of the imbalance through the admission events
            ev = out["events"][0][:out["n_events"][0]]
            assert st[orc.ST["I_after"]] == st[orc.ST["I_before"]] - int(sum(e["score"] for e in ev))
        oc.advance(1)
    assert len(placed) > 100


def test_non_anticipative(orc):
    """Assignments of a step do not depend on the output lengths of waiting requests."""
    for seed in range(20):
        cfg, init, arr = wl.random_case(seed, N=3, G=5, B=6, max_wait=20, H=0 if seed % 2 else 2,
                                        R_max=3, gate_pfin=0.0)
        a = _mk(orc, cfg, init).route_step(arr)["assign"]
        arr2 = wl.Arrivals(arr.count, arr.s, (arr.o * 7 + 3).astype(np.int32), arr.id, arr.pred)
        b = _mk(orc, cfg, init).route_step(arr2)["assign"]
        assert (a == b).all()


def test_h0_float_path_equals_br0(orc):
    """BR-H at H = 0 with (alpha, beta) = (1, G) makes the same decisions as BR-0 (Sec. 4.1)."""
    for seed in range(30):
        cfg, init, arr = wl.random_case(seed, N=4, G=int(3 + seed % 6), B=8, max_wait=24, H=0, R_max=4,
                                        tie_heavy=bool(seed % 3 == 0))
        a = _mk(orc, cfg, init).route_step(arr)
        b = _mk(orc, cfg, init, force_float=True).route_step(arr)
        assert (a["assign"] == b["assign"]).all()
        assert (a["F"].astype(np.float64) == b["F"].astype(np.float64)).all()
        assert (a["best_g"] == b["best_g"]).all() and (a["best_i"] == b["best_i"]).all()


def test_slot_limit_and_conservation_random(orc):
    for seed in range(40):
        H = [0, 2, 4][seed % 3]
        cfg, init, arr = wl.random_case(seed, N=4, G=int(2 + seed % 7), B=10, max_wait=32, H=H, R_max=4,
                                        fill=0.6, tie_heavy=bool(seed % 4 == 0), gate_pfin=0.0)
        oc = _mk(orc, cfg, init)
        L0, n0 = oc.L.copy(), oc.n.copy()
        out = oc.route_step(arr)
        for i in range(cfg.n_inst):
            qn = int(out["stats"][i, orc.ST["qlen"]])
            asg = out["assign"][i, :qn]
            s = np.clip(arr.s[i, :qn], 1, wl.MAX_S)
            for g in range(cfg.G):
                assert oc.n[i, g] == n0[i, g] + (asg == g).sum() <= cfg.B
                assert oc.L[i, g] == L0[i, g] + s[asg == g].sum() == oc.kv[i, g, :oc.n[i, g]].sum()
            assert (out["assign"][i, qn:] == -1).all()
            # deferred requests keep arrival order
            assert oc.qs[i, :oc.qlen[i]].tolist() == s[asg < 0].tolist()


def test_queue_cap_drops_are_counted(orc):
    cfg = wl.RouteConfig(name="q", n_inst=1, G=2, B=1, max_wait=4)
    oc = _mk(orc, cfg, _init([1, 1], [[10], [10]], 1))
    out = oc.route_step(_arr([5, 6, 7, 8, 9, 10]))
    assert out["stats"][0, orc.ST["dropped"]] == 2 and oc.qlen[0] == 4
    assert oc.qs[0, :4].tolist() == [5, 6, 7, 8]
    out = oc.route_step(_arr([11]))
    assert out["stats"][0, orc.ST["dropped"]] == 1 and out["stats"][0, orc.ST["admitted"]] == 0


def test_token_watermark_filter(orc):
    # Watermark 100, loads (95, 40), three free slots each, Stage 1 only; waiting 70, 50, 8, 3.
    # w1 (lighter) may take s <= 60 -> 50; w0 may take s <= 5 -> 3; caps tie, w1 (90) lighter: s <= 10 -> 8;
    # then neither worker can take 70: both are dropped for the rest of the step.
    cfg = wl.RouteConfig(name="w", n_inst=1, G=2, B=4, max_wait=8, token_watermark=100, token_cap=97, S_greedy=0)
    oc = _mk(orc, cfg, _init([1, 1], [[95], [40]], 4))
    out = oc.route_step(_arr([70, 50, 8, 3]))
    assert out["assign"][0, :4].tolist() == [-1, 1, 1, 0]
    assert oc.L[0].tolist() == [98, 98]
    assert out["stats"][0, orc.ST["workers_dropped"]] == 2
    assert out["stats"][0, orc.ST["overcap"]] == 2          # both loads exceed the reporting cap 97
    assert oc.qlen[0] == 1 and oc.qs[0, 0] == 70


# ---- brute force on tiny instances -----------------------------------------------------

def _brute_min_imbalance(L, cap, s, k):
    G, R = len(L), len(s)
    best = None
    for choice in itertools.product(range(-1, G), repeat=R):
        if sum(c >= 0 for c in choice) != k:
            continue
        cnt = [0] * G
        LL = list(L)
        ok = True
        for i, c in enumerate(choice):
            if c >= 0:
                cnt[c] += 1
                LL[c] += s[i]
                if cnt[c] > cap[c]:
                    ok = False
                    break
        if not ok:
            continue
        I = G * max(LL) - sum(LL)
        best = I if best is None else min(best, I)
    return best


def test_brute_force_bound_tiny(orc):
    """Against every assignment that admits the same number of requests under the slot limits:
    the two-stage result can never beat the optimum of the paper's objective I = G M - sum L
    (the paper claims no optimality), and the gap stays moderate on random tiny instances."""
    rng = np.random.default_rng(123)
    gaps = []
    for t in range(150):
        G = int(rng.integers(2, 4))
        B = int(rng.integers(1, 4))
        R = int(rng.integers(1, 7))
        n = rng.integers(0, B + 1, G)
        kv = [rng.integers(10, 400, int(n[g])).tolist() for g in range(G)]
        s = rng.integers(5, 500, R).tolist()
        cfg = wl.RouteConfig(name="bf", n_inst=1, G=G, B=B, max_wait=8, R_max=int(rng.integers(1, 5)),
                             S_greedy=int(rng.integers(0, 5)))
        oc = _mk(orc, cfg, _init(n.tolist(), kv, B))
        L0 = oc.L[0].tolist()
        cap = (B - n).tolist()
        out = oc.route_step(_arr(s))
        k = int(out["stats"][0, orc.ST["admitted"]])
        assert k == min(sum(cap), R)
        I_star = _brute_min_imbalance(L0, cap, s, k)
        I_br = int(out["stats"][0, orc.ST["I_after"]])
        assert I_br >= I_star
        gaps.append((I_br - I_star) / (I_star + max(s)))
    assert np.mean(np.array(gaps) == 0) > 0.4          # optimal on a good share of tiny cases
    assert np.mean(gaps) < 0.5


def test_single_request_goes_to_lightest_worker(orc):
    """One waiting request, equal free slots everywhere: the best score is on the lightest worker,
    which is also the brute-force optimum."""
    rng = np.random.default_rng(3)
    for t in range(100):
        G = int(rng.integers(2, 7))
        B = 3
        kv = [rng.integers(10, 400, 2).tolist() for _ in range(G)]
        s = [int(rng.integers(5, 500))]
        for sg in (0, 100):       # through Stage 1 and through Stage 2
            cfg = wl.RouteConfig(name="one", n_inst=1, G=G, B=B, max_wait=4, S_greedy=sg)
            oc = _mk(orc, cfg, _init([2] * G, kv, B))
            L0 = oc.L[0].copy()
            out = oc.route_step(_arr(s))
            g = int(out["assign"][0, 0])
            assert L0[g] == L0.min()
            assert out["stats"][0, orc.ST["I_after"]] == _brute_min_imbalance(L0.tolist(), [1] * G, s, 1)


# ---- decode step: Sec. 2.2 ---------------------------------------------------------------

def test_advance_closed_form(orc):
    cfg = wl.RouteConfig(name="adv", n_inst=1, G=2, B=4, max_wait=4)
    st = _init([3, 2], [[10, 20, 30], [5, 7]], 4)
    st.rem[0, 0, :3] = [100, 100, 100]
    st.rem[0, 1, :2] = [2, 100]
    oc = _mk(orc, cfg, st)
    oc.advance(1)
    assert oc.L[0].tolist() == [63, 14] and oc.n[0].tolist() == [3, 2]
    oc.advance(1)                          # the request with two steps to go leaves after its second
    assert oc.n[0].tolist() == [3, 1] and oc.L[0].tolist() == [66, 9]
    assert oc.kv[0, 1, 0] == 9 and oc.rem[0, 1, 0] == 98
    oc.advance(10)
    assert oc.L[0].tolist() == [66 + 30, 19]


def test_request_lifetime_loads(orc):
    # admitted with prefill s and output o: contributes s, s+1, ..., s+o-1 at exactly o steps
    cfg = wl.RouteConfig(name="life", n_inst=1, G=1, B=2, max_wait=2)
    oc = _mk(orc, cfg)
    oc.route_step(_arr([100], o=[4]))
    seen = []
    for _ in range(6):
        seen.append(int(oc.L[0, 0]))
        oc.advance(1)
    assert seen == [100, 101, 102, 103, 0, 0]


# ---- horizon projection: Appendix "Short-horizon prediction interface" -----------------

@pytest.mark.parametrize("H,mode", [(5, 0), (80, 1)])
def test_projection_anchor_closed_form(orc, H, mode):
    """All c_hat = H (hazards zero, or the estimate given as H): L_g(k+h) = L_g(k) + h * |A_g|; row h = 0 is
    the current load."""
    cfg, init, _ = wl.random_case(4, N=3, G=6, B=12, max_wait=8, H=H, pred_mode=mode)
    init.pred[...] = float(H) if mode else 0.0
    oc = _mk(orc, cfg, init)
    pr = oc.project()
    h = np.arange(H + 1)[None, None, :]
    assert (pr["Lh"] == oc.L[:, :, None] + h * oc.n[:, :, None]).all()
    assert (pr["Mh"] == pr["Lh"].max(axis=1)).all()
    assert (pr["mh"] == pr["Mh"][:, None, :] - pr["Lh"]).all() and (pr["mh"] >= 0).all()
    assert (pr["minm"] == pr["mh"].min(axis=2)).all()


@pytest.mark.parametrize("H", [6, 80])
def test_projection_vs_true_future(orc, H):
    """With c_hat = min(r, H) the projection equals the true future load except that a request is
    kept for one offset longer (at h = r <= H): the documented conservative index convention."""
    cfg, init, _ = wl.random_case(9, N=2, G=4, B=16, max_wait=8, H=H, pred_mode=1)
    init.pred[..., 0] = np.minimum(init.rem, H)
    oc = _mk(orc, cfg, init)
    pr = oc.project()
    used = np.arange(cfg.B)[None, None, :] < init.n[:, :, None]
    fut = _mk(orc, cfg, init)
    for h in range(H + 1):
        extra = np.where(used & (init.rem == h), init.kv + h, 0).sum(axis=2)
        assert (pr["Lh"][:, :, h] == fut.L + (extra if h >= 1 else 0)).all(), h
        fut.advance(1)


def test_projection_informative_hazards_cut(orc):
    """A sharp classifier (hazard ~1 at the true remaining length) drops the request from the
    offsets beyond it; gate at 0.5 accepts it because p_fin is high."""
    H = 4
    cfg = wl.RouteConfig(name="cut", n_inst=1, G=1, B=2, max_wait=2, H=H, gate_pfin=0.5)
    st = wl.InitState(np.array([[2]], np.int32), np.array([[[100, 200]]], np.int32),
                      np.array([[[2, 50]]], np.int32), np.zeros((1, 1, 2, H), np.float32))
    st.pred[0, 0, 0] = [0.0, 1.0, 0.0, 0.0]       # surely ends at its 2nd step: c_hat = 2
    st.pred[0, 0, 1] = 0.0                         # never in window: c_hat = H
    pr = _mk(orc, cfg, st).project()
    assert pr["chat"][0, 0].tolist() == [2.0, 4.0]
    assert pr["Lh"][0, 0].tolist() == [300, 302, 304, 203, 204]


# ---- the loop bounds and tie rules taken where the paper leaves them open, each on a hand-worked case ----

def test_stage1_runs_only_while_free_slots_exceed_threshold(orc):
    # Alg. BR-0: the greedy stage runs while S_tot > S_greedy (strictly).  One worker with three free
    # slots, S_greedy = 2, three waiting: one greedy admission (3 > 2), then the refined stage (2 > 2 fails).
    cfg = wl.RouteConfig(name="thr", n_inst=1, G=1, B=3, max_wait=8, R_max=1, S_greedy=2)
    oc = _mk(orc, cfg, _init([0], [[]], 3))
    st = oc.route_step(_arr([5, 4, 3]))["stats"][0]
    assert st[orc.ST["admitted"]] == 3 and st[orc.ST["stage1"]] == 1 and st[orc.ST["stage2_pops"]] == 2


def test_equal_subset_scores_resolve_to_lowest_mask(orc):
    # window (4, 4), one free slot, margin 100: masks 0b01 and 0b10 both score 4 -> 0b01
    P = orc.params_from(wl.RouteConfig(name="t2", n_inst=1, G=2, B=4, max_wait=8, R_max=2))
    assert orc.best_subset(P, [100], 0, 1, [4, 4]) == (1, 4.0)
    # window (8, 4, 4), two free slots, margin 8, G = 2: {8} scores 8, {4,4} scores 8, {8,4} 12-2*4=4 -> {8}
    P3 = orc.params_from(wl.RouteConfig(name="t2", n_inst=1, G=2, B=4, max_wait=8, R_max=3))
    assert orc.best_subset(P3, [8], 0, 2, [8, 4, 4]) == (1, 8.0)


def test_equal_single_scores_resolve_to_lowest_sorted_position(orc):
    # one worker slot to fill in the greedy stage (S_greedy = 0).
    # (a) equal lengths: the earlier arrival goes first
    cfg = wl.RouteConfig(name="t3", n_inst=1, G=2, B=1, max_wait=8, R_max=1, S_greedy=0)
    oc = _mk(orc, cfg, _init([0, 1], [[], [50]], 1))
    out = oc.route_step(_arr([7, 7, 7], ids=[11, 12, 13]))
    assert out["assign"][0, :3].tolist() == [0, -1, -1]
    # (b) equal scores of different lengths: worker 0 has margin 6 against worker 1's load; with G = 2,
    # s = 4 scores 4 and s = 8 scores 8 - 2*2 = 4: the longer request is first in the sorted order
    oc = _mk(orc, cfg, _init([0, 1], [[], [6]], 1))
    out = oc.route_step(_arr([4, 8], ids=[21, 22]))
    assert out["assign"][0, :2].tolist() == [-1, 0]


def test_admitted_load_enters_every_horizon_offset(orc):
    # BR-H, H = 1, gamma = 0.5, (alpha, beta) = (1, G = 2): d = (1, 0.5), alpha*D = 1.5; greedy stage only.
    # Two empty workers with one slot each, waiting (10, 12).  Worker 0 (lowest index) has margins (0, 0):
    # 12 scores 18 - 2*(12 + 6) = -18, 10 scores 15 - 2*(10 + 5) = -15 -> takes 10.  The 10 tokens count at
    # offsets 0 and 1: envelope (10, 10), worker 1 has margins (10, 10) and 12 scores 18 - 2*(2 + 1) = 12.
    # (Were the admitted load added at offset 0 only, the margin at offset 1 would be 0 and the score 2.)
    kw = dict(n_inst=1, G=2, max_wait=8, H=1, R_max=1, S_greedy=0, gamma=0.5, alpha=1.0, beta=2.0, pred_mode=1)
    oc = _mk(orc, wl.RouteConfig(name="a8", B=1, **kw), _init([0, 0], [[], []], 1))
    out = oc.route_step(_arr([10, 12], pred=np.ones((1, 2, 1), np.float32)), want_events=True)
    ev = out["events"][0][:out["n_events"][0]]
    assert [(int(e["g"]), int(e["delta"]), float(e["score"])) for e in ev] == [(0, 10, -15.0), (1, 12, 12.0)]
    # Two slots each, waiting (10, 12, 5, 4).  Worker 0, margins (0, 0): 4 scores 6 - 12 = -6, the best -> loads
    # (4, 0).  Worker 1 (two free slots), margins (4, 4): 12 -> -6, 10 -> -3, 5 -> 7.5 - 2*(1 + 0.5) = 4.5 ->
    # takes 5; loads (4, 5), envelope (5, 5).  One slot each: lighter worker 0, margins (1, 1): 12 -> -15,
    # 10 -> 15 - 2*(9 + 4.5) = -12 -> takes 10; envelope (14, 14).  Worker 1, margins (9, 9): 12 -> 18 - 2*4.5 = 9.
    oc = _mk(orc, wl.RouteConfig(name="a8b", B=2, **kw), _init([0, 0], [[], []], 2))
    out = oc.route_step(_arr([10, 12, 5, 4], pred=np.ones((1, 4, 1), np.float32)), want_events=True)
    ev = out["events"][0][:out["n_events"][0]]
    assert [(int(e["g"]), int(e["delta"]), float(e["score"])) for e in ev] == \
        [(0, 4, -6.0), (1, 5, 4.5), (0, 10, -12.0), (1, 12, 9.0)]


def test_c1_matches_stored_round(orc):
    """The smallest workload against tests/golden/c1_round.txt (written by tests/golden/make_c1_golden.py from
    the oracle alone): a change of the oracle's arithmetic or of the input generators shows up here."""
    import importlib.util
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_c1_golden", os.path.join(here, "make_c1_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    assert mod.compute() == open(os.path.join(here, "c1_round.txt")).read()


def test_brh_matches_stored_rounds(orc):
    """Two small BR-H rounds (H = 4 with hazards and gate; H = 80 with the two-stage pair) against
    tests/golden/brh_rounds.txt (written by tests/golden/make_brh_golden.py from the oracle alone): assignments,
    statistics, loads, the projection of one cluster and fp32 scores as bit patterns.  A change of the oracle's
    fp32 arithmetic, of its tie rules or of the input generators shows up here."""
    import importlib.util
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_brh_golden", os.path.join(here, "make_brh_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    assert mod.compute() == open(os.path.join(here, "brh_rounds.txt")).read()
