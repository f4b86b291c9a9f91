"""Pins for the oracle's pool-bypass dispatch (Appendix "Pool-bypass deployment path for BR-0")."""
import numpy as np

from paper_2605_06113_amd import workloads as wl
from tests.test_oracle_round import _arr, _init, _mk


def test_hand_worked_bypass(orc):
    # loads (100, 40), one request each, B = 3; arrivals 50, 30, 20 in order.
    # 50: margins (0, 60): F_0 = 50 - 2*50 = -50, F_1 = 50          -> worker 1, loads (100, 90)
    # 30: margins (0, 10): F_0 = -30, F_1 = 30 - 2*20 = -10         -> worker 1, loads (100, 120), now full
    # 20: M = 120, only worker 0 has a slot: F_0 = 20 (margin 20)   -> worker 0, loads (120, 120)
    cfg = wl.RouteConfig(name="bp", n_inst=1, G=2, B=3, max_wait=4)
    oc = _mk(orc, cfg, _init([1, 1], [[100], [40]], 3))
    out = oc.route_bypass(_arr([50, 30, 20], o=[7, 8, 9]))
    assert out["assign"][0, :3].tolist() == [1, 1, 0]
    assert oc.L[0].tolist() == [120, 120] and oc.n[0].tolist() == [2, 3]
    assert oc.kv[0, 1, :3].tolist() == [40, 50, 30] and oc.rem[0, 1, 1:3].tolist() == [7, 8]
    st = out["stats"][0]
    assert st[orc.ST["admitted"]] == 3 and st[orc.ST["I_before"]] == 60 and st[orc.ST["I_after"]] == 0


def test_bypass_placement_minimises_imbalance(orc):
    """F_g(s) = -Delta I (Sec. 3.1): each placement is the eligible worker with the smallest
    imbalance after it, lowest index on ties; loads are the running (virtual) ones."""
    rng = np.random.default_rng(17)
    for t in range(60):
        G, B = int(rng.integers(1, 9)), int(rng.integers(1, 6))
        n = rng.integers(0, B + 1, G)
        kv = [rng.integers(1, 3000, int(n[g])).tolist() for g in range(G)]
        s = rng.integers(1, 4000, int(rng.integers(1, 20))).tolist()
        cfg = wl.RouteConfig(name="bp", n_inst=1, G=G, B=B, max_wait=4)
        oc = _mk(orc, cfg, _init(n.tolist(), kv, B))
        L, cnt = oc.L[0].copy(), n.copy()
        out = oc.route_bypass(_arr(s))
        queued = 0
        for a, sa in enumerate(s):
            cands = [g for g in range(G) if cnt[g] < B]
            got = int(out["assign"][0, a])
            if not cands:
                queued += 1
                assert got == (-1 if queued <= cfg.max_wait else -2)
                continue
            def I_after(g):
                L2 = L.copy()
                L2[g] += sa
                return G * L2.max() - L2.sum()
            best = min(cands, key=lambda g: (I_after(g), g))
            assert got == best, (t, a)
            L[best] += sa
            cnt[best] += 1
        assert oc.L[0].tolist() == L.tolist() and oc.n[0].tolist() == cnt.tolist()
        assert oc.qlen[0] == min(queued, cfg.max_wait)
        assert out["stats"][0, orc.ST["dropped"]] == max(queued - cfg.max_wait, 0)


def test_bypass_first_arrival_equals_snapshot_best_worker(orc):
    """On the untouched snapshot the bypass choice is the per-request reduction of the score matrix."""
    for seed in range(10):
        cfg, init, arr = wl.random_case(seed, N=4, G=6, B=8, max_wait=16, H=0, n_wait=5)
        ref = _mk(orc, cfg, init).route_step(arr)          # snapshot best_g
        one = wl.Arrivals(np.ones_like(arr.count), arr.s, arr.o, arr.id, None)
        out = _mk(orc, cfg, init).route_bypass(one)
        assert (out["assign"][:, 0] == ref["best_g"][:, 0]).all()
