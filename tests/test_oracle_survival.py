"""Pins for the empirical-survival estimator and the refresh rules (pred_mode 2):
Appendix "Estimator realizations" and "Refresh logic"."""
import numpy as np

from paper_2605_06113_amd import workloads as wl
from tests.test_oracle_round import _arr, _mk


def _cfg(H, gate=0.0, refresh=0, **kw):
    base = dict(name="sv", n_inst=1, G=2, B=4, max_wait=8, H=H, pred_mode=2, gate_pfin=gate,
                refresh_period=refresh)
    base.update(kw)
    return wl.RouteConfig(**base)


def test_survival_matches_cdf_definition(orc):
    rng = np.random.default_rng(3)
    for _ in range(300):
        H = int(rng.integers(1, 81))
        n = int(rng.integers(1, 400))
        hist = np.sort(rng.integers(1, 300, n)).astype(np.int32)
        gate = float(rng.choice([0.0, 0.5]))
        P = orc.params_from(_cfg(H, gate), hist=hist)
        for a in rng.integers(0, 320, 12):
            a = int(a)
            # F(x) = #{o_j <= x}/n; the ratio (F(a+H) - F(a)) / (1 - F(a)) taken on the counts, so that a
            # value exactly at the gate is not moved across it by the division by n
            nF = lambda x: int((hist <= x).sum())
            surv = n - nF(a)
            inwin = hist[(hist > a) & (hist <= a + H)]
            if surv > 0 and len(inwin):
                pf = (nF(a + H) - nF(a)) / surv
                mu = (inwin - a).mean()
            else:
                pf, mu = 0.0, 0.0
            c = (1 - pf) * H + pf * mu
            if gate > 0 and pf < gate:
                c = H
            c = min(max(c, 1.0), H)
            assert abs(orc.survival(P, a) - c) <= 2e-6 * H + 1e-6, (H, n, a)


def test_survival_is_mean_of_truncated_remainder(orc):
    """Two-stage identity, eq. (two-stage), on the empirical measure: with the gate off the composite
    equals the mean of min(o_j - a, H) over the history entries that outlive age a."""
    rng = np.random.default_rng(4)
    for _ in range(200):
        H = int(rng.integers(2, 41))
        hist = np.sort(rng.integers(1, 120, int(rng.integers(5, 300)))).astype(np.int32)
        P = orc.params_from(_cfg(H, 0.0), hist=hist)
        a = int(rng.integers(0, 100))
        alive = hist[hist > a]
        if len(alive) == 0:
            assert orc.survival(P, a) == float(H)
            continue
        ref = np.minimum(alive - a, H).mean()
        assert abs(orc.survival(P, a) - max(ref, 1.0)) <= 2e-6 * H + 1e-6


def test_survival_special_cases(orc):
    hist = np.array([3, 3, 5, 9, 20, 20, 20, 100], np.int32)
    P = orc.params_from(_cfg(4, 0.0), hist=hist)
    assert orc.survival(P, 100) == 4.0 and orc.survival(P, 500) == 4.0      # outlived the history
    assert orc.survival(P, 30) == 4.0                                        # nothing ends in the window
    # age 16: survivors {20,20,20,100}; window (16,20] holds three with remainder 4: p=0.75, mu=4 -> 4
    assert orc.survival(P, 16) == 4.0
    # age 1: survivors all 8; window (1,5] holds 3,3,5: p=3/8, mu=(2+2+4)/3 -> (5/8)*4 + (3/8)*(8/3) = 3.5
    assert orc.survival(P, 1) == 3.5
    Pg = orc.params_from(_cfg(4, 0.5), hist=hist)
    assert orc.survival(Pg, 1) == 4.0                                        # p_fin 0.375 < 0.5: anchor H
    assert orc.survival(Pg, 16) == 4.0
    # age 2: survivors all 8, window (2,6] = {3,3,5}: same p; age 17..19 window hits the three 20s
    assert orc.survival(P, 19) == (1 - 0.75) * 4 + 0.75 * 1.0               # = 1.75


def test_refresh_schedule_hand_worked(orc):
    """H = 4, Delta T = 2.  History {3,3,5,9,20,20,20,100}.  One request admitted at step 0:
    query at age 0: window (0,4] = {3,3}: p = 2/8, mu = 3 -> c = 0.75*4 + 0.25*3 = 3.75.
    token 1: since 1 < 2: c = 2.75.   token 2: since 2 -> query at age 2: window (2,6] = {3,3,5},
    p = 3/8, mu = (1+1+3)/3 -> c = 2.5 + 0.625 = 3.125, since 0.   token 3: c = 2.125.
    token 4: query at age 4: survivors {5,9,20,20,20,100}, window (4,8] = {5}: p = 1/6, mu = 1
    -> c = (5/6)*4 + 1/6 = 3.5."""
    hist = np.array([3, 3, 5, 9, 20, 20, 20, 100], np.int32)
    cfg = _cfg(4, 0.0, refresh=2, G=1, B=2)
    oc = _mk(orc, cfg, hist=hist)
    oc.route_step(_arr([100], o=[50]))
    seen = [oc.pred[0, 0, 0].tolist()]
    for _ in range(4):
        oc.advance(1)
        seen.append(oc.pred[0, 0, 0].tolist())
    c2 = float(np.float32(np.float32(0.625) * np.float32(4.0)) + np.float32(np.float32(0.375) * (np.float32(5.0) / np.float32(3.0))))
    c4 = float(np.float32(np.float32(1.0) - np.float32(1.0) / np.float32(6.0)) * np.float32(4.0) + np.float32(1.0) / np.float32(6.0))
    assert seen[0] == [3.75, 0.0, 0.0]
    assert seen[1] == [2.75, 1.0, 1.0]
    assert seen[2][1:] == [2.0, 0.0] and abs(seen[2][0] - 3.125) < 1e-6 and abs(seen[2][0] - c2) < 1e-6
    assert seen[3][1:] == [3.0, 1.0] and abs(seen[3][0] - 2.125) < 1e-6
    assert seen[4][1:] == [4.0, 0.0] and abs(seen[4][0] - c4) < 1e-6 and abs(seen[4][0] - 3.5) < 1e-6


def test_floor_crossing_triggers_refresh(orc):
    # Delta T = 100 (no periodic refresh in this test).  Estimate at age 0 is 1.75 (history below);
    # after one token it would be 0.75 < 1: the estimator is queried at once, at age 1.
    hist = np.array([1, 1, 1, 50], np.int32)          # age 0: p = 3/4, mu = 1 -> 0.25*4 + 0.75 = 1.75
    cfg = _cfg(4, 0.0, refresh=100, G=1, B=2)
    oc = _mk(orc, cfg, hist=hist)
    oc.route_step(_arr([10], o=[50]))
    assert oc.pred[0, 0, 0].tolist() == [1.75, 0.0, 0.0]
    oc.advance(1)                                       # age 1: survivors {50}, nothing in window -> 4
    assert oc.pred[0, 0, 0].tolist() == [4.0, 1.0, 0.0]
    oc.advance(1)
    assert oc.pred[0, 0, 0].tolist() == [3.0, 2.0, 1.0]


def test_projection_uses_maintained_estimate(orc):
    hist = np.array([3, 3, 5, 9, 20, 20, 20, 100], np.int32)
    cfg = _cfg(4, 0.0, refresh=2, G=1, B=2)
    oc = _mk(orc, cfg, hist=hist)
    oc.route_step(_arr([100], o=[50]))
    oc.advance(1)                                       # kv 101, c_hat 2.75: offsets 0..2 count
    pr = oc.project()
    assert pr["chat"][0, 0, 0] == 2.75
    assert pr["Lh"][0, 0].tolist() == [101, 102, 103, 0, 0]
