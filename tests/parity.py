"""Shared comparison helpers: HIP path (through the C ABI) vs the CPU oracle."""
import numpy as np

from oracle import br_oracle
from paper_2605_06113_amd import binding

SCORE_RTOL = 1e-5   # fp32 horizon scores; integer results must be bit-exact


def compare_outputs(ref, out, cfg, tag=""):
    assert np.array_equal(out["stats"], ref["stats"]), f"{tag} stats\n{out['stats'][:2]}\n{ref['stats'][:2]}"
    assert np.array_equal(out["assign"], ref["assign"]), f"{tag} assign"
    assert np.array_equal(out["assign_id"], ref["assign_id"]), f"{tag} assign_id"
    qn = ref["stats"][:, br_oracle.ST["qlen"]]
    if "best_g" in out and "best_g" in ref:
        assert np.array_equal(out["best_g"], ref["best_g"]), f"{tag} best_g"
        assert np.array_equal(out["best_i"], ref["best_i"]), f"{tag} best_i"
    if "F" in out and "F" in ref:
        for i in range(cfg.n_inst):
            a, b = out["F"][i, :qn[i]], ref["F"][i, :qn[i]]
            if cfg.H == 0:
                assert np.array_equal(a, b), f"{tag} F inst {i}"
            else:
                np.testing.assert_allclose(a, b, rtol=SCORE_RTOL, atol=0, err_msg=f"{tag} F inst {i}")


def compare_state(oc, st, cfg, tag=""):
    assert np.array_equal(st["L"], oc.L), f"{tag} L"
    assert np.array_equal(st["n"], oc.n), f"{tag} n"
    assert np.array_equal(st["qlen"], oc.qlen), f"{tag} qlen"
    used = np.arange(cfg.B)[None, None, :] < oc.n[:, :, None]
    assert np.array_equal(st["kv"][used], oc.kv[used]), f"{tag} kv"
    assert np.array_equal(st["rem"][used], oc.rem[used]), f"{tag} rem"
    inq = np.arange(cfg.max_wait)[None, :] < oc.qlen[:, None]
    for k in ("qs", "qo", "qid"):
        assert np.array_equal(st[k][inq], getattr(oc, k)[inq]), f"{tag} {k}"
    if oc.P:
        assert np.array_equal(st["pred"][used], oc.pred[used]), f"{tag} pred"
    if oc.Pq:
        assert np.array_equal(st["qpred"][inq], oc.qpred[inq]), f"{tag} qpred"


def compare_prep(ref, st, tag=""):
    for k in ("Lh", "Mh", "mh", "minm"):
        assert np.array_equal(st[k], ref[k]), f"{tag} {k}"


def run_pair(cfg, init, arr, matrix=True, tag=""):
    """One round (+ one decode step) on both sides; returns (oracle, router) for further steps."""
    oc = br_oracle.OracleCluster(cfg, init)
    r = binding.Router(cfg, init)
    ref = oc.route_step(arr, want_prep=cfg.H > 0)
    out = r.route_step(arr, matrix=matrix)
    if cfg.H > 0:
        compare_prep(ref, r.state(), tag)     # projection buffers still hold the step-start values
    compare_outputs(ref, out, cfg, tag)
    compare_state(oc, r.state(), cfg, tag + " after route")
    oc.advance(1)
    r.advance(1)
    compare_state(oc, r.state(), cfg, tag + " after advance")
    return oc, r
