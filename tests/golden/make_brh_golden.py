"""Writes tests/golden/brh_rounds.txt: the oracle's result for two small BR-H rounds (seeded random snapshots,
three clusters each): H = 4 with a hazard per offset and the p_fin gate at 0.5, and H = 80 with the two stages
(p_fin, mu_rem) supplied per request.  Assignments, statistics, loads after the round and after one decode step,
the projected loads of cluster 0 and the fp32 scores of its first waiting request as bit patterns.  Calls only
the oracle and the seeded input generators; run from the repository root:  python tests/golden/make_brh_golden.py"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import br_oracle  # noqa: E402
from paper_2605_06113_amd import workloads as wl  # noqa: E402

CASES = (("h4", dict(seed=4040, N=3, G=5, B=10, max_wait=40, H=4, fill=0.6, gate_pfin=0.5)),
         ("h80", dict(seed=8080, N=3, G=6, B=12, max_wait=48, H=80, fill=0.6, pred_mode=3, gate_pfin=0.5, gamma=0.97)))


def case_inputs(kw):
    kw = dict(kw)
    return wl.random_case(kw.pop("seed"), **kw)


def compute():
    lines = []
    for tag, kw in CASES:
        cfg, init, arr = case_inputs(kw)
        oc = br_oracle.OracleCluster(cfg, init)
        out = oc.route_step(arr, want_prep=True)
        ints = lambda a: " ".join(str(int(x)) for x in np.asarray(a).ravel())
        lines += [f"# {tag}: {kw}",
                  f"{tag}.assign " + ints(out["assign"]),
                  f"{tag}.best_g " + ints(out["best_g"]),
                  f"{tag}.best_i " + ints(out["best_i"]),
                  f"{tag}.stats " + ints(out["stats"][:, :12]),
                  f"{tag}.L " + ints(oc.L),
                  f"{tag}.n " + ints(oc.n),
                  f"{tag}.Lh0 " + ints(out["Lh"][0]),
                  f"{tag}.F0bits " + ints(np.asarray(out["F"][0, 0], np.float32).view(np.int32))]
        oc.advance(1)
        lines += [f"{tag}.L1 " + ints(oc.L), f"{tag}.n1 " + ints(oc.n)]
    return "\n".join(lines) + "\n"


if __name__ == "__main__":
    with open(os.path.join(ROOT, "tests", "golden", "brh_rounds.txt"), "w") as f:
        f.write(compute())
