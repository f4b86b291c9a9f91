#!/usr/bin/env python3
"""Benchmark of the BalanceRoute route-step path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: one scheduling
round (score matrix reductions + two-stage assignment; horizon projection when H > 0) followed
by one decode step, on the batched throughput workload: 4096 independent BR-0 clusters, G=16,
B=144, 256 waiting requests and 128 active requests per worker each.  Every timed step runs on
its own copy of the cluster state (prepared before the timed region), so all steps do identical
work on data that is resident in HBM but not warm in cache.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# integer vector peak: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz, one int32 op per lane per clock
ALU_INT_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# HBM KiB per launch on this workload from rocprofv3 --pmc (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, see
# profiles/bench_c4_kernels.md); an entry is None when its kernel changed after the counters were taken
LDS_PEAK_GBS = 256 * 128 * 2.4          # 256 CUs x 128 B per clock x 2.4 GHz
LDS_INSTS_PER_WAVE = 236.1              # br_k_route4 (c4), rocprofv3 --pmc SQ_INSTS_LDS / SQ_WAVES
TRAFFIC_KIB = {"assign+advance": 2.0 * 43722.6 + 92343.4,   # br_k_route4<true>: reductions + round + decode step
               "assign": 2.0 * 6773.5 + 21800.9, "advance": 2.0 * 37923.5 + 74527.1}


def cpu_baseline(cfg, init, arr, min_seconds=10.0):
    """The oracle as it stands, single thread, on the same workload (repeated whole batches)."""
    from oracle import br_oracle
    pairs = 0
    decisions = 0
    elapsed = 0.0
    reps = 0
    while elapsed < min_seconds and reps < 50:
        oc = br_oracle.OracleCluster(cfg, init)
        t0 = time.perf_counter()
        out = oc.route_step(arr, want_scores=True)
        oc.advance(1)
        elapsed += time.perf_counter() - t0
        pairs += int(out["stats"][:, br_oracle.ST["qlen"]].sum()) * cfg.G
        decisions += int(out["stats"][:, br_oracle.ST["admitted"]].sum())
        reps += 1
    return dict(value=pairs / elapsed, unit="pairs/s", cores=1, kind="oracle",
                sample=f"{reps} x the full batch of {cfg.n_inst} instances (route + decode step), "
                       f"{elapsed:.1f} s of single-thread CPU time",
                decisions_per_s=decisions / elapsed)


def latency_run(steps, device, deployed=False):
    """Host wall-clock per round of one instance.  Default: the BR-H stress shape (G=64, H=8, queue cap 2048).
    deployed: the setting of the paper's dispatch-overhead measurement (Sec. 6.4: G=8, R_max=4, H=80), the
    estimate kept by the library with the empirical-survival estimator, workers near full."""
    import torch
    from paper_2605_06113_amd import binding, workloads as wl
    if deployed:
        cfg = wl.config("c5", G=8, B=64, max_wait=256, H=80, R_max=4, pred_mode=2, token_watermark=0,
                        token_cap=0, arrival_rate=0.7, arrival_rate_hi=2.0, init_active_per_worker=56,
                        init_kv_lo=256, init_kv_hi=8192, init_rem_lo=1, init_rem_hi=1024, seed=4100)
        hist = wl.output_history(cfg, 8000)
        init = wl.initial_state(cfg)
        label = ("paper's dispatch-overhead setting: BR-H H=80, G=8, R_max=4, B=64, queue cap 256, estimate maintained "
                 "from an 8000-length history (refresh every 40 tokens, gate 0.5), MMPP arrivals 0.7/2.0, one instance")
    else:
        cfg, hist, init = wl.config("c5"), None, None   # the paper's p_fin gate at its default
        label = "c5 shape: BR-H H=8, G=64, B=96, queue cap 2048, MMPP arrivals 60/300, one instance"
    tr = wl.arrival_trace(cfg, steps)
    warm = binding.Router(cfg, init, device=device, hist=hist)   # untimed: loads the kernels this shape uses
    for k in range(3):
        warm.route_step(tr.step(k), matrix=False)
        warm.advance(1)
    warm.close()
    r = binding.Router(cfg, init, device=device, hist=hist)
    P = r.P
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a, dt), device=device)
    count, s, o, ids = t(tr.count, np.int32), t(tr.s, np.int32), t(tr.o, np.int32), t(tr.id, np.int32)
    pred = t(tr.pred, np.float32) if r.Pq else None
    out = r.alloc_outputs(scores=True, matrix=False)
    ostruct = r.out_struct(out)
    import ctypes as C
    lat = np.zeros(steps)
    qlen = np.zeros(steps, np.int64)
    cap = int(tr.s.shape[-1])
    torch.cuda.synchronize()
    for k in range(steps):
        a = binding.Arrivals(count=count[k].data_ptr(), s=s[k].data_ptr(), o=o[k].data_ptr(),
                             id=ids[k].data_ptr(), pred=pred[k].data_ptr() if r.Pq else None, arr_cap=cap, pad=0)
        t0 = time.perf_counter()
        rc = r.lib.br_route_step(r.ctx, C.byref(a), C.byref(ostruct))
        r.stream.synchronize()
        lat[k] = time.perf_counter() - t0
        assert rc == 0
        r.advance(1)
    torch.cuda.synchronize()
    st = out["stats"].cpu().numpy()
    steady = lat[steps // 2:]
    res = dict(workload=label,
               steps=steps, p50_us=float(np.percentile(lat, 50) * 1e6), p99_us=float(np.percentile(lat, 99) * 1e6),
               max_us=float(lat.max() * 1e6), steady_p50_us=float(np.percentile(steady, 50) * 1e6),
               steady_p99_us=float(np.percentile(steady, 99) * 1e6), final_qlen=int(st[0, binding.ST["deferred"]]))
    if deployed:
        state = r.state()
        res["mean_us"] = float(lat.mean() * 1e6)
        res["final_active"] = int(state["n"].sum())
        # context only: another machine, the production trace, a Python dispatcher (Sec. 6.4)
        res["paper_dispatch_ms"] = dict(p50=1.20, mean=1.34, p99=2.77)
    r.close()
    return res


def brh_run(device, steps=5, warmup=1, gate=None, deployed=False):
    """Batched BR-H round (horizon projection + scores + assignment) and decode step:
    4096 clusters of the c3 shape (G=32, B=96, H=4), 76 active requests per worker, 256 waiting.
    deployed: 2048 clusters at the horizon and window of Sec. 6 (H=80, R_max=4, G=8; B=64, 48 active per
    worker, 256 waiting), the estimate maintained by the library."""
    import torch
    from paper_2605_06113_amd import binding, workloads as wl
    over = {} if gate is None else dict(gate_pfin=gate)
    per_worker = 48 if deployed else 76
    if deployed:
        cfg = wl.config("c3", n_inst=2048, G=8, B=64, max_wait=256, H=80, R_max=4, pred_mode=2, token_watermark=0,
                        token_cap=0, init_active_per_worker=per_worker, init_kv_lo=256, init_kv_hi=8192, init_rem_lo=1,
                        init_rem_hi=1024, init_waiting=256, seed=2100)
        hist = wl.output_history(cfg, 8000)
    else:
        cfg = wl.config("c3", n_inst=4096, **over, token_watermark=0, token_cap=0, init_active_per_worker=per_worker,
                        init_kv_lo=256, init_kv_hi=8192, init_rem_lo=1, init_rem_hi=1024, init_waiting=256)
        hist = None
    init, arr = wl.initial_state(cfg), wl.initial_waiting(cfg)
    routers = [binding.Router(cfg, init, device=device, hist=hist) for _ in range(steps + warmup)]
    darr = binding.DeviceArrivals(arr, device, routers[0].Pq)
    out = routers[0].alloc_outputs(scores=True, matrix=False)
    torch.cuda.synchronize()
    for r in routers[:warmup]:
        r.route_advance_device(darr, out, 1)
    torch.cuda.synchronize()
    for r in routers[warmup:]:
        r.profile(True)
    t0 = time.perf_counter()
    for r in routers[warmup:]:
        r.route_advance_device(darr, out, 1)   # projection, scores, assignment + decode step
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    stats = out["stats"].cpu().numpy()
    admitted = int(stats[:, binding.ST["admitted"]].sum())
    qn = int(stats[:, binding.ST["qlen"]].sum())
    kern = {k: [0.0, 0] for k in binding.KERNEL_NAMES}
    for r in routers[warmup:]:
        for k, (ms, c) in r.profile_read().items():
            kern[k][0] += ms
            kern[k][1] += c
    for r in routers:
        r.close()
    N, G, H, P = cfg.n_inst, cfg.G, cfg.H, routers[0].P
    active = N * G * per_worker
    bytes_k = dict(project=active * (4 + 4 * P) + N * G * 4 + N * (H + 1) * 4 * (2 * G + 1) + N * G * 4,
                   advance=(active + admitted) * 16 + N * G * 16)
    res = dict(workload=f"{N} clusters: BR-H H={H}, G={G}, B={cfg.B}, R_max={cfg.R_max}, {per_worker} active per worker, "
                        f"256 waiting; p_fin gate {cfg.gate_pfin}" + ("; estimate maintained by the library" if deployed else ""),
               ms_per_step=elapsed / steps * 1e3, pairs_per_s=qn * G * steps / elapsed,
               decisions_per_s=admitted * steps / elapsed, kernels={})
    for k, (ms, c) in kern.items():
        if c == 0 or k == "init":
            continue
        e = dict(avg_ms=ms / c, launches=c)
        if k in bytes_k:
            gbs = bytes_k[k] / (ms / c * 1e-3) / 1e9
            e.update(bound="hbm", achieved_GBs=gbs, frac=gbs / HBM_PEAK_GBS)
        res["kernels"][k] = e
    return res


def replay_run(device, n_inst=1024, steps=300):
    """Replayed decode steps, batched: n_inst independent copies (own arrival streams) of the BR-0 replay
    shape (G=16, B=96, Poisson(40) arrivals per step, queue cap 256), from empty clusters; every step is one
    br_route_advance (round + decode step in one launch, no score outputs)."""
    import torch
    from paper_2605_06113_amd import binding, workloads as wl
    cfg = wl.config("c2", n_inst=n_inst)
    tr = wl.arrival_trace(cfg, steps)
    r = binding.Router(cfg, None, device=device)
    t = lambda a: torch.as_tensor(np.ascontiguousarray(a, np.int32), device=device)
    count, s, o, ids = t(tr.count), t(tr.s), t(tr.o), t(tr.id)
    cap = int(tr.s.shape[-1])
    out = r.alloc_outputs(scores=False)
    stats_all = torch.zeros((steps, n_inst, binding.NSTATS), dtype=torch.int64, device=device)  # one row block per step
    import ctypes as C
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        a = binding.Arrivals(count=count[k].data_ptr(), s=s[k].data_ptr(), o=o[k].data_ptr(), id=ids[k].data_ptr(),
                             pred=None, arr_cap=cap, pad=0)
        out["stats"] = stats_all[k]
        ostruct = r.out_struct(out)
        rc = r.lib.br_route_advance(r.ctx, C.byref(a), C.byref(ostruct), 1)
        assert rc == 0
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    st_all = stats_all.cpu().numpy()
    admitted = int(st_all[:, :, binding.ST["admitted"]].sum())
    pairs = int(st_all[:, :, binding.ST["qlen"]].sum())
    st = st_all[-1]
    res = dict(workload=f"{n_inst} instances of the c2 shape replayed from empty for {steps} decode steps "
                        "(BR-0, G=16, B=96, Poisson(40) arrivals, queue cap 256), one br_route_advance per step",
               ms_per_step=elapsed / steps * 1e3, instance_steps_per_s=n_inst * steps / elapsed,
               decisions_per_s=admitted / elapsed, pairs_per_s=pairs * cfg.G / elapsed,
               final_mean_queue=float(st[:, binding.ST["deferred"]].mean()))
    r.close()
    return res


def bypass_run(device, cfg, init, arr, steps=6, warmup=2):
    """Pool-bypass dispatch (BR-0) of the same batch: 256 arrivals per cluster placed one by one."""
    import torch
    from paper_2605_06113_amd import binding
    routers = [binding.Router(cfg, init, device=device) for _ in range(steps + warmup)]
    darr = binding.DeviceArrivals(arr, device, 0)
    out = dict(assign=torch.empty((cfg.n_inst, darr.arr_cap), dtype=torch.int32, device=device),
               stats=torch.empty((cfg.n_inst, binding.NSTATS), dtype=torch.int64, device=device))
    for r in routers[:warmup]:
        r.route_bypass_device(darr, out)
    torch.cuda.synchronize()
    for r in routers[warmup:]:
        r.profile(True)
    t0 = time.perf_counter()
    for r in routers[warmup:]:
        r.route_bypass_device(darr, out)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    st = out["stats"].cpu().numpy()
    placed = int(st[:, binding.ST["admitted"]].sum())
    ms = cnt = 0
    for r in routers[warmup:]:
        m, c = r.profile_read()["bypass"]
        ms += m
        cnt += c
    for r in routers:
        r.close()
    return dict(workload="c4 state, 256 arrivals per cluster dispatched one at a time (argmax_g over 16 workers each)",
                ms_per_call=elapsed / steps * 1e3, kernel_avg_ms=ms / max(cnt, 1), decisions_per_s=placed * steps / elapsed,
                pairs_per_s=int(st[:, binding.ST["qlen"]].sum()) * cfg.G * steps / elapsed)


def window_run(device, R_max=16, n_inst=1024, steps=4, warmup=1):
    """Stage 2 with a wide candidate window: the c4 cluster shape with R_max = 16 and S_greedy = 64 as in the
    main workload, so the last 64 free slots of a cluster (4 per worker) are filled by pops that search the
    subsets of at most 4 out of 16 requests."""
    import torch
    from paper_2605_06113_amd import binding, workloads as wl
    cfg = wl.config("c4", n_inst=n_inst, R_max=R_max, S_greedy=64)
    init, arr = wl.initial_state(cfg), wl.initial_waiting(cfg)
    routers = [binding.Router(cfg, init, device=device) for _ in range(steps + warmup)]
    darr = binding.DeviceArrivals(arr, device, 0)
    out = routers[0].alloc_outputs(scores=False)
    for r in routers[:warmup]:
        r.route_advance_device(darr, out, 1)
    torch.cuda.synchronize()
    for r in routers[warmup:]:
        r.profile(True)
    t0 = time.perf_counter()
    for r in routers[warmup:]:
        r.route_advance_device(darr, out, 1)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    st = out["stats"].cpu().numpy()
    ms = cnt = 0
    for r in routers[warmup:]:
        m, c = r.profile_read()["assign"]
        ms += m
        cnt += c
    for r in routers:
        r.close()
    pops, guard = int(st[:, binding.ST["stage2_pops"]].sum()), int(st[:, binding.ST["guard"]].sum())
    return dict(workload=f"{n_inst} clusters of the c4 shape with R_max={R_max}, S_greedy=64: round + decode step",
                ms_per_step=elapsed / steps * 1e3, assign_kernel_ms=ms / max(cnt, 1), stage2_pops=pops, guard_pops=guard,
                decisions_per_s=int(st[:, binding.ST["admitted"]].sum()) * steps / elapsed)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--latency-steps", type=int, default=10000,
                    help="decode steps of the single-instance latency replay (the stress shape runs 10000)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-every", type=int, default=4,
                    help="bracket the kernels of every n-th timed step with HIP events (per-kernel durations)")
    ap.add_argument("--two-calls", action="store_true",
                    help="time br_route_step + br_advance_decode instead of the fused br_route_advance")
    ap.add_argument("--no-two-calls-leg", action="store_true", help="skip the side measurement of the two-call step")
    ap.add_argument("--no-brh", action="store_true", help="skip the batched BR-H side measurement")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for scaling rocprofv3 byte counters)")
    ap.add_argument("--traffic-kib", type=float, default=None,
                    help="HBM KiB per launch of the dominant kernel from rocprofv3 --pmc runs, if known")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (instances shard across GPUs with no exchange); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_06113_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    device = "cuda:0"
    binding.load()

    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.int32, device=device)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cfg = wl.config("c4")
    init, arr = wl.initial_state(cfg), wl.initial_waiting(cfg)
    K, W = args.steps, args.warmup
    darr = binding.DeviceArrivals(arr, device, 0)

    def timed(fused):
        """W + K steps, each on its own copy of the cluster state; per-kernel HIP-event times from every n-th of the K."""
        routers = [binding.Router(cfg, init, device=device) for _ in range(K + W)]
        out = routers[0].alloc_outputs(scores=True, matrix=False)
        torch.cuda.synchronize()

        def step(r):
            if fused:
                r.route_advance_device(darr, out, 1)
            else:
                r.route_step_device(darr, out)
                r.advance(1)

        for r in routers[:W]:
            step(r)
        torch.cuda.synchronize()
        for r in routers[W::args.profile_every]:
            r.profile(True)       # HIP-event pairs around every kernel of these steps (each costs ~7 us of stream time)
        t0 = time.perf_counter()
        for r in routers[W:]:
            step(r)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        stats = out["stats"].cpu().numpy()
        kern = {k: [0.0, 0] for k in binding.KERNEL_NAMES}
        for r in routers[W:]:
            for k, (ms, c) in r.profile_read().items():
                kern[k][0] += ms
                kern[k][1] += c
        for r in routers:
            r.close()
        del routers, out
        return t1 - t0, stats, kern

    fused = not args.two_calls
    elapsed, stats, kern = timed(fused)
    admitted = int(stats[:, binding.ST["admitted"]].sum())
    qn = int(stats[:, binding.ST["qlen"]].sum())
    pairs_per_step = qn * cfg.G

    # algorithmic work per launch of each kernel
    N, G, B, Q = cfg.n_inst, cfg.G, cfg.B, cfg.max_wait
    occupied_after = N * G * 128 + admitted          # slots the decode step touches
    bytes_advance = occupied_after * 16 + N * G * 16  # kv, rem read + written; L, n read + written
    bytes_score = qn * 4 + qn * 4 + N * G * (8 + 4)   # s read, best_g written; L, n read, best_i written
    bytes_assign = qn * (4 + 4 + 4 + 4 + 4) + admitted * 8 + N * G * 16 + N * 16 * 8
    ops_assign = 4.0 * admitted * (Q)               # per admission: one score (4 int ops) per waiting slot

    def kernel_table(kern, fused):
        tab = {}
        for k, (ms, c) in kern.items():
            if c == 0:
                continue
            avg = ms / c
            e = dict(avg_ms=avg, launches=c)
            # on this workload the snapshot reductions ride in the assignment launch (br_k_route4); the fused
            # launch also streams the lists
            b_assign = bytes_assign + (qn * 4 + N * G * 4) + (bytes_advance if fused else 0)   # + outputs of the reductions
            o_assign = ops_assign + 4.0 * pairs_per_step
            if k == "advance":
                e.update(bound="hbm", achieved_GBs=bytes_advance / (avg * 1e-3) / 1e9,
                         frac=bytes_advance / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS)
            elif k == "score":
                e.update(bound="hbm", achieved_GBs=bytes_score / (avg * 1e-3) / 1e9,
                         frac=bytes_score / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS)
            elif k == "assign":
                e.update(bound="alu", achieved_Tops=o_assign / (avg * 1e-3) / 1e12,
                         frac=o_assign / (avg * 1e-3) / 1e12 / ALU_INT_PEAK_TOPS,
                         hbm_GBs=b_assign / (avg * 1e-3) / 1e9, includes_snapshot_reductions=True,
                         includes_decode_step=bool(fused))
            tab[k] = e
        return tab

    per_kernel = kernel_table(kern, fused)
    dom = max((k for k in per_kernel if k != "init"), key=lambda k: per_kernel[k]["avg_ms"])
    d = per_kernel[dom]
    if d["bound"] == "hbm":
        roofline = dict(bound="hbm", kernel=dom, achieved=d["achieved_GBs"], peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=d["frac"])
    else:
        roofline = dict(bound="alu", kernel=dom, achieved=d["achieved_Tops"], peak=ALU_INT_PEAK_TOPS, unit="TOP/s",
                        frac=d["frac"])
    kib = args.traffic_kib if args.traffic_kib is not None else TRAFFIC_KIB.get(dom + ("+advance" if fused else ""))
    roofline["traffic"] = None if kib is None else kib * 1024.0
    roofline["avg_launch_ms"] = d["avg_ms"]
    if dom == "assign":
        # LDS traffic of the round kernel: instructions per wave from rocprofv3 --pmc SQ_INSTS_LDS (profiles/), taken
        # as 64 lanes x 4 B each, against 128 B per clock and CU; the dependent chain lives in registers and DPP
        lds_bytes = LDS_INSTS_PER_WAVE * 64 * 4 * cfg.n_inst
        lds_gbs = lds_bytes / (d["avg_ms"] * 1e-3) / 1e9
        roofline["lds"] = dict(achieved_GBs=lds_gbs, peak_GBs=LDS_PEAK_GBS, frac=lds_gbs / LDS_PEAK_GBS,
                               insts_per_wave=LDS_INSTS_PER_WAVE)
    step_bytes = bytes_advance + bytes_score + bytes_assign
    ms_per_step = elapsed / K * 1e3

    res = dict(metric="F-score pairs/sec (batched route step + decode step); decisions/sec and single-instance "
                      "route-step latency alongside",
               value=pairs_per_step * K / elapsed, unit="pairs/s", n_gpus=1, steps=K, warmup=W,
               ms_per_step=ms_per_step, higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="int32", data="synthetic",
               config=dict(workload="c4: 4096 independent BR-0 instances, G=16, B=144, 256 waiting + 128 active "
                                    "per worker, one route step + one decode step",
                           n_inst=N, G=G, B=B, max_wait=Q, H=0, R_max=cfg.R_max, S_greedy=cfg.s_greedy,
                           parallelism="1 gpu"),
               decisions_per_s=admitted * K / elapsed,
               step_hbm_GBs=step_bytes / (ms_per_step * 1e-3) / 1e9,
               step_hbm_frac=step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
               entry="br_route_advance" if fused else "br_route_step + br_advance_decode",
               roofline=roofline, kernels=per_kernel)
    if fused and not args.no_two_calls_leg:
        e2, _, k2 = timed(False)
        res["two_calls"] = dict(entry="br_route_step + br_advance_decode", ms_per_step=e2 / K * 1e3,
                                pairs_per_s=pairs_per_step * K / e2, kernels=kernel_table(k2, False))
    if not args.no_brh:
        res["brh_batched"] = brh_run(device)
        res["brh_batched_gate_off"] = brh_run(device, gate=0.0)   # hazards live: no request counts at the last offset
        res["brh_batched_h80"] = brh_run(device, deployed=True)
        res["window16"] = window_run(device)
        res["bypass"] = bypass_run(device, cfg, init, arr)
        res["replay_batched"] = replay_run(device)
    if args.latency_steps > 0:
        res["latency"] = latency_run(args.latency_steps, device)
        res["latency_deployed"] = latency_run(min(args.latency_steps, 4000), device, deployed=True)
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg, init, arr)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
