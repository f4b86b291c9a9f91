"""br_route_step_static (the entry point for callers that cannot allocate: the partial results of the tiled
stage-one reductions live in a fixed device array inside the library) against br_route_step on twin contexts,
and both against the CPU oracle: two calls in a row, the second with a smaller input, then a smaller context
that finds the array full of the larger one's partial results."""
import sys

import numpy as np
import pytest

from oracle import br_oracle
from paper_2605_06113_amd import binding, workloads as wl
from tests.parity import compare_outputs, compare_state

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _static_step(r, arr, matrix=False):
    darr = binding.DeviceArrivals(arr, r.device, r.Pq) if arr is not None else None
    out = r.alloc_outputs(scores=True, matrix=matrix)
    rc = r.route_step_static_device(darr, out)
    assert rc == binding.BR_OK, rc
    r.stream.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


def _twin_rounds(tag, cfg, init, arrs):
    """The same rounds through both entry points and the oracle; outputs and state must agree bit for bit
    (fp32 scores are not written here: matrix off, which is what selects the tiled reductions)."""
    oc = br_oracle.OracleCluster(cfg, init)
    ra, rb = binding.Router(cfg, init), binding.Router(cfg, init)
    for k, arr in enumerate(arrs):
        _say(f"{tag}: call {k}, arrivals {arr.count.tolist() if arr is not None else None}")
        ref = oc.route_step(arr)
        a = ra.route_step(arr, matrix=False)
        b = _static_step(rb, arr)
        for key in ("assign", "assign_id", "stats", "best_g", "best_i"):
            assert np.array_equal(a[key], b[key]), f"{tag} call {k}: {key} differs between the two entry points"
        compare_outputs({kk: ref[kk] for kk in b}, b, cfg, f"{tag} call {k} vs oracle")
        # the valid part of the snapshot (lists up to n, queue up to qlen) through both entry points
        compare_state(oc, ra.state(), cfg, f"{tag} call {k} (br_route_step)")
        compare_state(oc, rb.state(), cfg, f"{tag} call {k} (br_route_step_static)")
        oc.advance(1), ra.advance(1), rb.advance(1)
    ra.close(), rb.close()


def test_static_scratch_entry_matches_route_step():
    # the single-instance stress shape: 32 request tiles x 4 worker groups of partial results
    cfg, init, big = wl.random_case(301, N=1, G=64, B=40, max_wait=2048, H=8, fill=0.7, n_wait=1500,
                                    gate_pfin=0.0, s_hi=32768)
    _, _, small = wl.random_case(302, N=1, G=64, B=40, max_wait=2048, H=8, n_wait=37, gate_pfin=0.0)
    _twin_rounds("H=8 G=64 Q=2048", cfg, init, [big, small, None])
    # a smaller context next: BR-0, three clusters, shorter queues, fewer workers (other layout of the same array)
    cfg, init, a1 = wl.random_case(303, N=3, G=16, B=24, max_wait=512, H=0, fill=0.6, n_wait=400)
    _, _, a2 = wl.random_case(304, N=3, G=16, B=24, max_wait=512, H=0, n_wait=9)
    _twin_rounds("BR-0 N=3 Q=512", cfg, init, [a1, a2])
    # the most clusters it serves, long horizon (partial results of the LDS-resident score)
    cfg, init, a1 = wl.random_case(305, N=16, G=9, B=12, max_wait=700, H=80, pred_mode=1, fill=0.5, n_wait=600)
    _, _, a2 = wl.random_case(306, N=16, G=9, B=12, max_wait=700, H=80, pred_mode=1, n_wait=50)
    _twin_rounds("H=80 N=16 Q=700", cfg, init, [a1, a2])


def test_static_scratch_entry_limit_and_no_events():
    cfg, init, arr = wl.random_case(307, N=17, G=8, B=12, max_wait=600, H=0, n_wait=300)
    r = binding.Router(cfg, init)
    out = r.alloc_outputs(scores=True, matrix=False)
    for v in out.values():
        v.fill_(-7)
    rc = r.route_step_static_device(binding.DeviceArrivals(arr, r.device, r.Pq), out)
    assert rc == binding.BR_ELIMIT
    r.stream.synchronize()
    assert all(bool((v == -7).all()) for v in out.values())      # nothing was enqueued
    r.close()
    # with profiling on, the static entry point still creates no event pair: nothing is recorded for it
    cfg, init, arr = wl.random_case(308, N=2, G=16, B=12, max_wait=600, H=0, n_wait=300)
    r = binding.Router(cfg, init)
    r.profile(True)
    _static_step(r, arr)
    assert all(c == 0 for _, c in r.profile_read().values())
    r.route_step(arr, matrix=False)
    assert r.profile_read()["assign"][1] == 1
    r.close()
