"""Pins for the oracle's score functions and the in-window contribution.

Everything here checks oracle/br_oracle.c against what the paper and the mathematics
fix, computed independently in numpy / Python (fp64 or exact integers).
"""
import itertools
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


# ---- BR-0 score: Sec. 3.1, eq. (br0-Fscore) -------------------------------------------

def test_br0_golden_breakpoints(orc):
    rows = [tuple(map(int, ln.split())) for ln in open(os.path.join(HERE, "golden", "br0_score_breakpoints.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 20
    for G, m, d, F in rows:
        assert orc.score_br0(G, m, d) == F, (G, m, d)


@pytest.mark.parametrize("G", [2, 3, 4, 8, 16, 64])
def test_br0_shape(orc, G):
    rng = np.random.default_rng(G)
    for m in [0, 1, 7, 1000, 65536] + list(rng.integers(0, 100000, 5)):
        m = int(m)
        assert orc.score_br0(G, m, 0) == 0
        assert orc.score_br0(G, m, m) == m                       # value at the kink
        assert orc.score_br0(G, m, m + 1) == m - (G - 1)         # first overflow unit
        for d in rng.integers(0, max(m, 1), 5):                  # safe regime: slope +1
            d = int(d)
            if d + 1 <= m:
                assert orc.score_br0(G, m, d + 1) - orc.score_br0(G, m, d) == 1
        for d in rng.integers(m, m + 50000, 5):                  # overflow: slope -(G-1)
            d = int(d)
            assert orc.score_br0(G, m, d + 1) - orc.score_br0(G, m, d) == -(G - 1)
        if G > 1 and (G * m) % (G - 1) == 0:                     # zero crossing at G m / (G-1)
            assert orc.score_br0(G, m, G * m // (G - 1)) == 0


def test_br0_score_is_imbalance_drop(orc):
    """F_g(Q) = I_before - I_after with I = G max(L) - sum(L) (Sec. 3.1), exact in integers."""
    rng = np.random.default_rng(11)
    for _ in range(2000):
        G = int(rng.integers(1, 65))
        L = rng.integers(0, 500000, G).astype(np.int64)
        if rng.random() < 0.3:
            L[rng.integers(0, G)] = L.max()        # ties at the top
        g = int(rng.integers(0, G))
        d = int(rng.integers(0, 200000))
        I0 = G * L.max() - L.sum()
        L2 = L.copy()
        L2[g] += d
        I1 = G * L2.max() - L2.sum()
        assert orc.score_br0(G, int(L.max() - L[g]), d) == I0 - I1


# ---- horizon score: Sec. 4.1, eq. (brh-Fscore) ----------------------------------------

def _f64_horizon(alpha, beta, gamma, m, d):
    H = len(m) - 1
    dv = np.float64(gamma) ** np.arange(H + 1)
    return alpha * dv.sum() * d - beta * (np.maximum(d - np.asarray(m, np.float64), 0.0) * dv).sum()


def test_brh_reduces_to_br0_at_h0(orc):
    rng = np.random.default_rng(5)
    for _ in range(2000):
        G = int(rng.integers(1, 65))
        m = int(rng.integers(0, 300000))
        d = int(rng.integers(0, 262144))
        f = orc.score_brh(0, 1.0, float(G), 0.7, [m], d)
        assert f == float(orc.score_br0(G, m, d))     # exact: all values below 2^24


def test_brh_matches_fp64_definition(orc):
    rng = np.random.default_rng(6)
    for _ in range(3000):
        H = int(rng.integers(0, 81))
        alpha = float(np.float32(rng.uniform(0.5, 2.0)))
        beta = float(np.float32(rng.uniform(0.0, 64.0)))
        gamma = float(np.float32(rng.uniform(0.3, 1.0)))
        m = rng.integers(0, 100000, H + 1)
        d = int(rng.integers(0, 262144))
        f = orc.score_brh(H, alpha, beta, gamma, m, d)
        ref = _f64_horizon(alpha, beta, gamma, m, d)
        scale = alpha * (H + 1) * d + beta * (H + 1) * d + 1.0
        assert abs(f - ref) <= 2e-6 * scale, (H, alpha, beta, gamma, d)


def test_brh_score_is_discounted_imbalance_drop(orc):
    """With (alpha, beta) = (1, G) the horizon score is minus the change of
    sum_h gamma^h (G M_h - sum_g L_g(k+h)) when Delta is added at every offset."""
    rng = np.random.default_rng(7)
    for _ in range(500):
        G = int(rng.integers(2, 33))
        H = int(rng.integers(1, 9))
        gamma = float(np.float32(rng.uniform(0.4, 1.0)))
        Lh = rng.integers(0, 400000, (G, H + 1)).astype(np.float64)
        g = int(rng.integers(0, G))
        d = int(rng.integers(1, 100000))
        dv = np.float64(gamma) ** np.arange(H + 1)
        J0 = (dv * (G * Lh.max(axis=0) - Lh.sum(axis=0))).sum()
        L2 = Lh.copy()
        L2[g] += d
        J1 = (dv * (G * L2.max(axis=0) - L2.sum(axis=0))).sum()
        m = (Lh.max(axis=0) - Lh[g]).astype(np.int64)
        f = orc.score_brh(H, 1.0, float(G), gamma, m, d)
        assert abs(f - (J0 - J1)) <= 1e-5 * (abs(J0 - J1) + G * (H + 1) * d)


def test_brh_equal_margins_gamma_one(orc):
    rng = np.random.default_rng(8)
    for _ in range(500):
        H = int(rng.integers(1, 9))
        m = int(rng.integers(0, 4096))        # small enough that every product is exact in fp32
        d = int(rng.integers(0, 8192))
        alpha, beta = 1.0, float(rng.integers(1, 17))
        f = orc.score_brh(H, alpha, beta, 1.0, [m] * (H + 1), d)
        assert f == (H + 1) * (alpha * d - beta * max(d - m, 0))


def test_brh_concave_piecewise_linear(orc):
    """Horizon-safe regime is linear; at most H+1 kinks, located at the margins; concave."""
    rng = np.random.default_rng(9)
    for _ in range(50):
        H = int(rng.integers(1, 9))
        m = np.sort(rng.integers(10, 200, H + 1))
        alpha, beta, gamma = 1.0, 8.0, 0.5        # dyadic parameters: fp32 arithmetic stays exact
        f = np.array([orc.score_brh(H, alpha, beta, gamma, m, d) for d in range(0, 260)], np.float64)
        D = sum(gamma ** h for h in range(H + 1))
        lo = int(m.min())
        assert np.all(f[:lo + 1] == alpha * D * np.arange(lo + 1))
        slope = np.diff(f)
        second = np.diff(slope)
        assert np.all(second <= 0)
        kinks = set((np.nonzero(second)[0] + 1).tolist())
        assert kinks <= set(int(x) for x in m) and len(kinks) <= H + 1


# ---- in-window contribution: eqs. (two-stage) / (composite) ---------------------------

def _two_stage_f64(p):
    """(1 - p_fin) H + p_fin mu_rem from the pmf of r implied by hazards p (fp64)."""
    H = len(p)
    p = np.asarray(p, np.float64)
    surv = np.concatenate([[1.0], np.cumprod(1.0 - p)])      # S_0..S_H
    pmf = surv[:-1] * p                                      # P(r = j), j = 1..H
    pfin = pmf.sum()
    if pfin == 0.0:
        return float(H), 0.0
    mu = (np.arange(1, H + 1) * pmf).sum() / pfin
    return (1.0 - pfin) * H + pfin * mu, pfin


def test_chat_equals_two_stage_composite(orc):
    rng = np.random.default_rng(12)
    for _ in range(3000):
        H = int(rng.integers(1, 81))
        kind = rng.integers(0, 3)
        if kind == 0:
            p = rng.beta(2, 50, H)
        elif kind == 1:
            p = rng.uniform(0, 1, H)
        else:
            p = np.full(H, 0.02)
            p[rng.integers(0, H)] = 0.9
        p = p.astype(np.float32)
        ref, _ = _two_stage_f64(p)
        c = orc.chat(H, 0, 0.0, p)                            # gate off
        assert abs(c - max(ref, 1.0)) <= 1e-5 * H


def test_chat_from_two_stage_pair(orc):
    """pred_mode 3: eq. (composite) on a supplied (p_fin, mu_rem): c_hat = (1 - p_fin) H + p_fin mu_rem, gate on
    p_fin, floor 1, clip H; against fp64 and at the corners."""
    rng = np.random.default_rng(14)
    for _ in range(3000):
        H = int(rng.integers(1, 129))
        pf, mu = float(np.float32(rng.uniform(0, 1))), float(np.float32(rng.uniform(0, H + 1)))
        c = orc.chat(H, 3, 0.0, [pf, mu])
        ref = min(max((1.0 - pf) * H + pf * mu, 1.0), float(H))
        assert abs(c - ref) <= 1e-5 * H
        gate = 0.5
        cg = orc.chat(H, 3, gate, [pf, mu])
        assert cg == (float(H) if pf < gate else c)
    assert orc.chat(80, 3, 0.0, [0.0, 7.0]) == 80.0          # surely not finishing in the window: the anchor H
    assert orc.chat(80, 3, 0.0, [1.0, 7.0]) == 7.0           # surely finishing: the regressor's value
    assert orc.chat(80, 3, 0.0, [1.0, 0.25]) == 1.0          # floor
    assert orc.chat(80, 3, 0.0, [0.5, 200.0]) == 80.0        # clip
    assert orc.chat(80, 3, 0.5, [0.5, 10.0]) == 45.0         # at the gate the estimate is used: 0.5 * 80 + 0.5 * 10


def test_chat_special_cases(orc):
    for H in [1, 2, 4, 8, 80]:
        assert orc.chat(H, 0, 0.0, np.zeros(H)) == float(H)            # never finishes in window
        p = np.zeros(H)
        p[0] = 1.0
        assert orc.chat(H, 0, 0.0, p) == 1.0                           # finishes next step
        assert orc.chat(H, 0, 0.5, p) == 1.0                           # gate passes (p_fin = 1)
        p = np.full(H, 0.01)                                           # p_fin small: gate -> anchor H
        _, pfin = _two_stage_f64(p)
        if pfin < 0.5:
            assert orc.chat(H, 0, 0.5, p) == float(H)
            if H >= 2:
                assert orc.chat(H, 0, 0.0, p) < float(H)
        # direct c_hat: floor 1 and clip to H
        assert orc.chat(H, 1, 0.5, [0.25]) == 1.0
        assert orc.chat(H, 1, 0.5, [H + 5.0]) == float(H)
        if H >= 2:
            assert orc.chat(H, 1, 0.5, [1.5]) == 1.5


def test_chat_gate_boundary(orc):
    # p_fin exactly 0.5 passes the gate (accepted when p_fin >= 0.5)
    assert orc.chat(4, 0, 0.5, [0.5, 0.0, 0.0, 0.0]) == 1.0 + 0.5 * 3
    assert orc.chat(4, 0, 0.5, [0.25, 0.0, 0.0, 0.0]) == 4.0


# ---- Stage-2 subset search: Appendix "Bit-set subset selection" -----------------------

def _reachable(win, kmax):
    sums = {}
    for r in range(1, kmax + 1):
        for comb in itertools.combinations(range(len(win)), r):
            sums.setdefault(sum(win[i] for i in comb), []).append(comb)
    return sums


@pytest.mark.parametrize("H", [0, 4])
def test_subset_search_is_max_over_reachable_sums(orc, H):
    from paper_2605_06113_amd.workloads import RouteConfig
    rng = np.random.default_rng(21 + H)
    for _ in range(300):
        G = int(rng.integers(2, 17))
        R_max = int(rng.integers(1, 9))
        cfg = RouteConfig(name="t", n_inst=1, G=G, B=8, max_wait=8, H=H, R_max=R_max, gamma=0.5)
        P = orc.params_from(cfg)
        w = int(rng.integers(1, R_max + 1))
        win = sorted(rng.integers(1, 3000, w).tolist(), reverse=True)
        cap = int(rng.integers(1, 9))
        m = rng.integers(0, 6000, H + 1)
        mask, f = orc.best_subset(P, m, 0, cap, win)
        sums = _reachable(win, min(cap, R_max))
        if H == 0:
            scores = {d: orc.score_br0(G, int(m[0]), d) for d in sums}
        else:
            scores = {d: orc.score_brh(H, cfg.alpha, cfg.beta_eff, cfg.gamma, m, d) for d in sums}
        best = max(scores.values())
        assert f == best
        chosen = sum(win[b] for b in range(w) if mask >> b & 1)
        assert scores[chosen] == best and bin(mask).count("1") <= min(cap, R_max)
        if H == 0:
            # two-probe rule: the optimum is the largest reachable sum <= m or the smallest above it
            below = [d for d in sums if d <= m[0]]
            above = [d for d in sums if d > m[0]]
            probes = ([max(below)] if below else []) + ([min(above)] if above else [])
            assert best == max(scores[d] for d in probes)


@pytest.mark.parametrize("H", [0, 6])
def test_subset_search_matches_bitset_reduction(orc, H):
    """Appendix "Bit-set subset selection": F_g(Q) depends on Q only through its sum, so the optimum over subsets of
    at most k requests is the optimum of F over the sums reachable with 1..k requests.  The reachable sets are
    built here by the shift-OR recurrence dp[j] |= dp[j-1] << s_i on Python integers (j descending), for windows
    of up to 16 requests, and the exhaustive search must return that optimum with a subset that attains it."""
    from paper_2605_06113_amd.workloads import RouteConfig
    rng = np.random.default_rng(121 + H)
    for _ in range(60):
        G = int(rng.integers(2, 33))
        R_max = int(rng.integers(9, 17))
        cfg = RouteConfig(name="t", n_inst=1, G=G, B=32, max_wait=32, H=H, R_max=R_max, gamma=0.8)
        P = orc.params_from(cfg)
        w = int(rng.integers(R_max - 2, R_max + 1))
        win = sorted(rng.integers(1, 2500, w).tolist(), reverse=True)
        cap = int(rng.integers(1, 20))
        kmax = min(cap, R_max)
        m = rng.integers(0, 12000, H + 1)
        dp = [0] * (kmax + 1)
        dp[0] = 1
        for s in win:
            for j in range(kmax, 0, -1):
                dp[j] |= dp[j - 1] << s
        reach = 0
        for j in range(1, kmax + 1):
            reach |= dp[j]
        sums = [b for b in range(reach.bit_length()) if reach >> b & 1]
        if H == 0:
            best = max(orc.score_br0(G, int(m[0]), d) for d in sums)
        else:
            best = max(orc.score_brh(H, cfg.alpha, cfg.beta_eff, cfg.gamma, m, d) for d in sums)
        mask, f = orc.best_subset(P, m, 0, cap, win)
        assert f == best
        chosen = sum(win[b] for b in range(w) if mask >> b & 1)
        assert reach >> chosen & 1 and 1 <= bin(mask).count("1") <= kmax
        fc = orc.score_br0(G, int(m[0]), chosen) if H == 0 else orc.score_brh(H, cfg.alpha, cfg.beta_eff, cfg.gamma, m, chosen)
        assert fc == best


# ---- wide windows: the subset search by reachable sums (Appendix "Bit-set subset selection") -------------------

def _wide_case(rng, w, tie_heavy, H):
    from paper_2605_06113_amd.workloads import RouteConfig
    G = int(rng.integers(1, 33))
    R_max = int(rng.integers(max(w, 1), 33))
    cfg = RouteConfig(name="t", n_inst=1, G=G, B=64, max_wait=64, H=H, R_max=R_max, gamma=float(rng.choice([0.64, 0.9, 1.0])),
                      token_watermark=int(rng.choice([0, 0, 9000])))
    if tie_heavy:
        win = sorted(rng.choice([64, 128, 192, 256], w).tolist(), reverse=True)
        m = rng.integers(0, 1500, H + 1)
    else:
        win = sorted(rng.integers(1, int(rng.choice([40, 2500, 9000])), w).tolist(), reverse=True)
        m = rng.integers(0, int(rng.choice([300, 12000, 60000])), H + 1)
    cap = int(rng.integers(1, 40))
    L_g = int(rng.integers(0, 5000))
    return cfg, win, m, cap, L_g


@pytest.mark.parametrize("H", [0, 3])
def test_reachable_sum_search_equals_scan_of_all_masks(orc, H):
    """Wherever both apply the two searches return the same subset and score: windows of 1..16 requests against
    the scan the round uses there, windows of 17..20 against the same scan run over all 2^w masks.  Equal lengths
    (many subsets per sum, many sums per score) exercise the lowest-mask rule."""
    rng = np.random.default_rng(400 + H)
    for case in range(150):
        w = int(rng.integers(1, 17)) if case < 120 else int(rng.integers(17, 21))
        cfg, win, m, cap, L_g = _wide_case(rng, w, tie_heavy=case % 3 == 0, H=H)
        P = orc.params_from(cfg)
        a = orc.best_subset(P, m, L_g, cap, win)
        b = orc.best_subset_reach(P, m, L_g, cap, win)
        assert (a[0] & 0xFFFFFFFF, a[1]) == b, (case, w, win, m.tolist(), cap, a, b)


def test_reachable_sum_search_32_requests_lowest_mask_by_halves(orc):
    """Windows of 32 requests, BR-0: the optimum over reachable sums by the shift-OR recurrence on Python integers,
    and the lowest mask that attains it found independently by splitting the window into two halves of 16 (upper
    half masks in ascending order, the lowest matching lower-half mask from a table)."""
    from paper_2605_06113_amd.workloads import RouteConfig
    rng = np.random.default_rng(77)
    for case in range(12):
        G = int(rng.integers(2, 33))
        w = 32
        cfg = RouteConfig(name="t", n_inst=1, G=G, B=64, max_wait=64, H=0, R_max=32)
        P = orc.params_from(cfg)
        win = sorted((rng.choice([64, 128, 192, 256], w) if case % 2 else rng.integers(1, 3000, w)).tolist(), reverse=True)
        cap = int(rng.integers(1, 12))
        kmax = min(cap, 32)
        m = int(rng.integers(0, 20000))
        mask, f = orc.best_subset_reach(P, [m], 0, cap, win)
        dp = [0] * (kmax + 1)
        dp[0] = 1
        for s in win:
            for j in range(kmax, 0, -1):
                dp[j] |= dp[j - 1] << s
        reach = dp[kmax] >> 1 << 1            # at most kmax requests (dp[j] contains dp[j-1]: dp[0] = {0} stays in all)
        for j in range(1, kmax):
            reach |= dp[j]
        sums = [b for b in range(1, reach.bit_length()) if reach >> b & 1]
        best = max(orc.score_br0(G, m, d) for d in sums)
        assert f == best
        targets = {d for d in sums if orc.score_br0(G, m, d) == best}
        # lower half: for every (number of requests, sum) the lowest 16-bit mask
        lo_w, hi_w = np.array(win[:16]), np.array(win[16:])
        masks = np.arange(1 << 16)
        bits = (masks[:, None] >> np.arange(16)) & 1
        lo_sum, hi_sum, pop = bits @ lo_w, bits @ hi_w, bits.sum(1)
        table = {}
        for mk in range((1 << 16) - 1, -1, -1):
            table[(int(pop[mk]), int(lo_sum[mk]))] = mk          # descending: the lowest mask is written last
        found = None
        for u in range(1 << 16):
            if pop[u] > kmax:
                continue
            cands = [table.get((p, d - int(hi_sum[u]))) for d in targets for p in range(0, kmax - int(pop[u]) + 1)]
            cands = [c for c in cands if c is not None and (c or u)]
            if cands:
                found = (u << 16) | min(cands)
                break
        assert found == mask, (case, hex(found), hex(mask))


def test_reachable_sum_table_ends_at_its_bound(orc):
    """Subsets whose sum exceeds the table's bound (131071) are not candidates: 17 requests of 32768 tokens, room
    for 5, a margin that would take them all: three requests (98304) are the most the table holds."""
    from paper_2605_06113_amd.workloads import RouteConfig
    cfg = RouteConfig(name="t", n_inst=1, G=4, B=64, max_wait=64, H=0, R_max=17)
    P = orc.params_from(cfg)
    mask, f = orc.best_subset_reach(P, [10 ** 6], 0, 5, [32768] * 17)
    assert (mask, f) == (0b111, 98304.0)
    mask, f = orc.best_subset_reach(P, [10 ** 6], 0, 5, [32768] + [100] * 16)     # 32768 + 4 x 100 fits
    assert (mask, f) == (0b11111, 33168.0)
