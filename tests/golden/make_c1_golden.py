"""Writes tests/golden/c1_round.txt: the oracle's result for the smallest workload (BR-0, one cluster, G = 4,
20 active and 32 waiting requests, seed 0) after one scheduling round and one decode step.  Calls only the
oracle and the seeded input generators; run from the repository root:  python tests/golden/make_c1_golden.py"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import br_oracle  # noqa: E402
from paper_2605_06113_amd import workloads as wl  # noqa: E402


def compute():
    cfg = wl.config("c1")
    oc = br_oracle.OracleCluster(cfg, wl.initial_state(cfg))
    out = oc.route_step(wl.initial_waiting(cfg))
    st = out["stats"][0]
    lines = ["# c1: assign[i] for the 32 arrivals in arrival order (-1 = deferred)",
             "assign " + " ".join(str(int(x)) for x in out["assign"][0, :32]),
             "# per-request best worker and per-worker best request on the step-start snapshot",
             "best_g " + " ".join(str(int(x)) for x in out["best_g"][0, :32]),
             "best_i " + " ".join(str(int(x)) for x in out["best_i"][0]),
             "# admitted deferred dropped stage1 stage2_pops guard overcap I_before I_after spread",
             "stats " + " ".join(str(int(st[k])) for k in range(10)),
             "# loads and request counts right after the round",
             "L " + " ".join(str(int(x)) for x in oc.L[0]),
             "n " + " ".join(str(int(x)) for x in oc.n[0])]
    oc.advance(1)
    lines += ["# loads and request counts after one decode step",
              "L1 " + " ".join(str(int(x)) for x in oc.L[0]),
              "n1 " + " ".join(str(int(x)) for x in oc.n[0])]
    return "\n".join(lines) + "\n"


if __name__ == "__main__":
    with open(os.path.join(ROOT, "tests", "golden", "c1_round.txt"), "w") as f:
        f.write(compute())
