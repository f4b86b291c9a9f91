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
LDS_PEAK_GBS = 256 * 128 * 2.4          # 256 CUs x 128 B per clock x 2.4 GHz
PROFILE_MD = os.path.join(ROOT, "profiles", "bench_c4_kernels.md")


def source_hash():
    """sha256 over the kernel sources and the C header: counters in profiles/ are valid for exactly one value."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2605_06113_amd", "csrc")
    for f in sorted(os.listdir(csrc)) + [os.path.join(ROOT, "include", "br.h")]:
        path = f if os.path.isabs(f) else os.path.join(csrc, f)
        h.update(os.path.basename(path).encode() + b"\0" + open(path, "rb").read())
    return h.hexdigest()


def profile_counters():
    """Counter figures of the rocprofv3 summary (lines `counter <name> <kernel> = <value>` of its last section),
    or {} when the sources have changed since they were collected (then they say nothing about these kernels)."""
    vals, sha = {}, None
    try:
        for line in open(PROFILE_MD):
            line = line.strip()
            if line.startswith("sources_sha256 = "):
                sha = line.split("=", 1)[1].strip()
            elif line.startswith("counter "):
                key, val = line[len("counter "):].rsplit("=", 1)
                vals[key.strip()] = float(val)
    except OSError:
        return {}
    return vals if sha == source_hash() else {}


def host_info():
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        gcc = __import__("subprocess").check_output(["gcc", "--version"], text=True).splitlines()[0]
    except Exception:
        gcc = "gcc (version unknown)"
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return dict(nproc=os.cpu_count(), usable_cpus=usable, cpu_model=model,
                compiler=gcc + " -O2 -ffp-contract=off (oracle/br_oracle.c, one thread per instance stream)")


def _take_instances(obj, lo, hi):
    import dataclasses
    return type(obj)(**{f.name: (None if getattr(obj, f.name) is None else getattr(obj, f.name)[lo:hi])
                        for f in dataclasses.fields(obj)})


_PARTS = None


def _oracle_batch(c, i, a):
    from oracle import br_oracle
    oc = br_oracle.OracleCluster(c, i)
    t0 = time.perf_counter()
    out = oc.route_step(a, want_scores=True)
    oc.advance(1)
    dt = time.perf_counter() - t0
    return dt, int(out["stats"][:, br_oracle.ST["qlen"]].sum()) * c.G, int(out["stats"][:, br_oracle.ST["admitted"]].sum())


def _oracle_part(k):
    return _oracle_batch(*_PARTS[k])


def cpu_baseline(cfg, init, arr, min_seconds=8.0):
    """The oracle as it stands on the host cores of this machine, same arrays as the GPU.  Primary figure: the
    single-threaded oracle fanned over the usable cores, one slice of the instances per thread (instances are
    independent; the C code runs outside the interpreter lock).  Beside it the single-thread rate, and the oracle's
    per-step latency on the one-instance configurations."""
    import dataclasses
    from oracle import br_oracle
    from paper_2605_06113_amd import workloads as wl
    info = host_info()

    batch = _oracle_batch
    # (i) one thread, whole batches
    pairs = decisions = reps = 0
    elapsed = 0.0
    while elapsed < min_seconds and reps < 50:
        dt, p, d = batch(cfg, init, arr)
        elapsed += dt
        pairs += p
        decisions += d
        reps += 1
    single = dict(value=pairs / elapsed, unit="pairs/s", cores=1, decisions_per_s=decisions / elapsed,
                  us_per_instance_step=elapsed / (reps * cfg.n_inst) * 1e6,
                  sample=f"{reps} x the full batch of {cfg.n_inst} instances (route + decode step), {elapsed:.1f} s")

    # (ii) all usable cores (os.sched_getaffinity, at most 16): the same single-threaded oracle in T worker
    # processes, one contiguous slice of the instances each (this process never touches the GPU, so it may fork)
    import multiprocessing as mp
    T = max(1, min(info["usable_cpus"], 16, cfg.n_inst))
    cuts = [cfg.n_inst * k // T for k in range(T + 1)]
    global _PARTS
    _PARTS = [(dataclasses.replace(cfg, n_inst=cuts[k + 1] - cuts[k]), _take_instances(init, cuts[k], cuts[k + 1]),
               _take_instances(arr, cuts[k], cuts[k + 1])) for k in range(T)]
    pairs = decisions = reps = 0
    wall = 0.0
    with mp.get_context("fork").Pool(T) as pool:
        pool.map(_oracle_part, range(T))          # untimed: workers start, the oracle library loads in each
        while wall < min_seconds / 2 and reps < 200:
            t0 = time.perf_counter()
            res = pool.map(_oracle_part, range(T))
            wall += time.perf_counter() - t0
            pairs += sum(r[1] for r in res)
            decisions += sum(r[2] for r in res)
            reps += 1
    allc = dict(value=pairs / wall, unit="pairs/s", cores=T, decisions_per_s=decisions / wall,
                sample=f"{reps} x the full batch, instances split over {T} processes of one thread each, {wall:.1f} s wall")

    # (iii) per-step latency of the oracle on the single-instance configurations (wall-clock of orc_route_step)
    per_cfg = {}
    for name, steps in (("c1", 1), ("c2", 2000), ("c3", 1000), ("c5", 3000)):
        c = wl.config(name)
        lat = []
        if name == "c1":
            i1, a1 = wl.initial_state(c), wl.initial_waiting(c)
            for _ in range(200):
                oc = br_oracle.OracleCluster(c, i1)
                t0 = time.perf_counter()
                oc.route_step(a1, want_scores=False)
                lat.append(time.perf_counter() - t0)
        else:
            tr = wl.arrival_trace(c, steps)
            oc = br_oracle.OracleCluster(c)
            for k in range(steps):
                a = tr.step(k)
                t0 = time.perf_counter()
                oc.route_step(a, want_scores=False)
                lat.append(time.perf_counter() - t0)
                oc.advance(1)
        lat = np.array(lat) * 1e6
        per_cfg[name] = dict(steps=len(lat), mean_us=float(lat.mean()), p50_us=float(np.percentile(lat, 50)),
                             p99_us=float(np.percentile(lat, 99)),
                             note="200 repeats of the one round" if name == "c1" else
                             (f"first {steps} of {c.steps} decode steps" if steps < c.steps else "all decode steps"))
    return dict(value=allc["value"], unit="pairs/s", cores=T, kind="oracle",
                sample=allc["sample"] + "; workload: the bench's own batch (c4), route + decode step",
                decisions_per_s=allc["decisions_per_s"], single_thread=single, per_step_latency=per_cfg, **info)


def latency_run(steps, device, deployed=False, name="c5"):
    """Host wall-clock per round of one instance.  Default: the BR-H stress shape (G=64, H=8, queue cap 2048);
    name: another of the single-instance replay configurations (c2, c3).
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
        cfg, hist, init = wl.config(name), None, None   # the paper's p_fin gate at its default
        label = {"c5": "c5 shape: BR-H H=8, G=64, B=96, queue cap 2048, MMPP arrivals 60/300, one instance",
                 "c3": "c3: BR-H H=4, G=32, B=96, queue cap 512, Poisson(80) arrivals, one instance",
                 "c2": "c2: BR-0, G=16, B=96, queue cap 256, Poisson(40) arrivals, one instance"}[name]
        steps = min(steps, cfg.steps)
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
               mean_us=float(lat.mean() * 1e6), max_us=float(lat.max() * 1e6), steady_p50_us=float(np.percentile(steady, 50) * 1e6),
               steady_p99_us=float(np.percentile(steady, 99) * 1e6), final_qlen=int(st[0, binding.ST["deferred"]]))
    if deployed:
        state = r.state()
        res["final_active"] = int(state["n"].sum())
        # context only: another machine, the production trace, a Python dispatcher (Sec. 6.4)
        res["paper_dispatch_ms"] = dict(p50=1.20, mean=1.34, p99=2.77)
    r.close()
    return res


def brh_run(device, steps=8, warmup=1, gate=None, deployed=False):
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
    for r in routers[warmup::4]:
        r.profile(True)       # event pairs on every fourth timed step only (a pair costs ~7 us of stream time)
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


def bypass_run(device, cfg, init, arr, steps=8, warmup=2):
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
    for r in routers[warmup::4]:
        r.profile(True)       # event pairs on every fourth timed step only (a pair costs ~7 us of stream time)
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


def window_run(device, R_max=16, n_inst=1024, steps=8, warmup=1, S_greedy=64):
    """Stage 2 with a wide candidate window: the c4 cluster shape with R_max = 16 (every subset mask) or 32 (the
    reachable sums of Appendix "Bit-set subset selection"); with S_greedy = 64 as in the main workload the last 64
    free slots of a cluster (4 per worker) are filled by pops that search subsets of at most 4 requests of the
    window, with S_greedy = 512 every admission goes through Stage 2 (up to 16 requests per pop)."""
    import torch
    from paper_2605_06113_amd import binding, workloads as wl
    cfg = wl.config("c4", n_inst=n_inst, R_max=R_max, S_greedy=S_greedy)
    init, arr = wl.initial_state(cfg), wl.initial_waiting(cfg)
    routers = [binding.Router(cfg, init, device=device) for _ in range(steps + warmup)]
    darr = binding.DeviceArrivals(arr, device, 0)
    out = routers[0].alloc_outputs(scores=False)
    for r in routers[:warmup]:
        r.route_advance_device(darr, out, 1)
    torch.cuda.synchronize()
    for r in routers[warmup::4]:
        r.profile(True)       # event pairs on every fourth timed step only (a pair costs ~7 us of stream time)
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
    return dict(workload=f"{n_inst} clusters of the c4 shape with R_max={R_max}, S_greedy={S_greedy}: round + decode step",
                ms_per_step=elapsed / steps * 1e3, assign_kernel_ms=ms / max(cnt, 1), stage2_pops=pops, guard_pops=guard,
                decisions_per_s=int(st[:, binding.ST["admitted"]].sum()) * steps / elapsed)


def quality_run(device, name="c2", steps=2000):
    """Trace-mean imbalance (max - min load per step, Sec. 6.1) of the comparison policies, BR-0 and BR-H on one
    replay workload, all through the C ABI on the same synthetic trace; BR-H runs with c_hat = min(remaining
    steps, H) kept by the caller in the workspace (the paper's "BR-H oracle" configuration).  Per-step statistics
    stay on the device until the end.  Qualitative comparison: synthetic traces, not the paper's numbers."""
    import dataclasses
    import torch
    from paper_2605_06113_amd import binding, workloads as wl
    base = wl.config(name, token_watermark=0, token_cap=0)
    steps = min(steps, base.steps)
    H = base.H if base.H > 0 else 8
    flat = dataclasses.replace(base, H=0, pred_mode=0)
    res = {}
    for policy in ("random", "rr", "p2c", "jsq", "br0", "brh"):
        cfg = dataclasses.replace(base, H=H, pred_mode=1) if policy == "brh" else flat
        tr = wl.arrival_trace(cfg, steps)
        r = binding.Router(cfg, None, device=device)
        t = lambda a, dt=np.int32: torch.as_tensor(np.ascontiguousarray(a, dt), device=device)
        count, s, o, ids = t(tr.count), t(tr.s), t(tr.o), t(tr.id)
        pred = t(np.minimum(tr.o, H)[..., None], np.float32) if policy == "brh" else None
        cap = int(tr.s.shape[-1])
        out = r.alloc_outputs(scores=False)
        stats_all = torch.zeros((steps, 1, binding.NSTATS), dtype=torch.int64, device=device)
        lay = r.layout
        import ctypes as C
        t0 = time.perf_counter()
        for k in range(steps):
            a = binding.Arrivals(count=count[k].data_ptr(), s=s[k].data_ptr(), o=o[k].data_ptr(), id=ids[k].data_ptr(),
                                 pred=pred[k].data_ptr() if pred is not None else None, arr_cap=cap, pad=0)
            out["stats"] = stats_all[k]
            ostruct = r.out_struct(out)
            if policy in binding.POLICY:
                rc = r.lib.br_route_baseline(r.ctx, C.byref(a), C.byref(ostruct), binding.POLICY[policy], 5)
            else:
                rc = r.lib.br_route_step(r.ctx, C.byref(a), C.byref(ostruct))
            assert rc == 0
            r.advance(1)
            if policy == "brh":
                r._view(lay.pred, (1, r.G, r.Bs, 1), "f32")[..., 0].copy_(r._view(lay.rem, (1, r.G, r.Bs)).clamp(max=H).float())
                r._view(lay.qpred, (1, r.Q, 1), "f32")[..., 0].copy_(r._view(lay.qo, (1, r.Q)).clamp(max=H).float())
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        st = stats_all.cpu().numpy()[:, 0]
        res[policy] = dict(mean_imbalance=float(st[steps // 5:, binding.ST["spread"]].mean()),
                           admitted=int(st[:, binding.ST["admitted"]].sum()), us_per_step=dt / steps * 1e6)
        r.close()
    return dict(workload=f"{name} shape, {steps} decode steps, one instance (G={base.G}, B={base.B}, queue cap {base.max_wait}); "
                         f"mean over the last four fifths of max - min load after each round; BR-H: H={H}, c_hat = min(remaining, H)",
                policies=res)


def c1_latency(device, reps=200):
    """The single BR-0 round of c1 (one instance, G=4, 32 waiting), repeated on fresh contexts."""
    import torch
    from paper_2605_06113_amd import binding, workloads as wl
    cfg = wl.config("c1")
    init, arr = wl.initial_state(cfg), wl.initial_waiting(cfg)
    darr = binding.DeviceArrivals(arr, device, 0)
    lat = []
    for k in range(reps + 3):
        r = binding.Router(cfg, init, device=device)
        out = r.alloc_outputs(scores=True, matrix=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        r.route_step_device(darr, out)
        r.stream.synchronize()
        if k >= 3:
            lat.append(time.perf_counter() - t0)
        r.close()
    lat = np.array(lat) * 1e6
    return dict(workload="c1: one BR-0 round, one instance, G=4, B=16, 20 active, 32 waiting", steps=reps,
                mean_us=float(lat.mean()), p50_us=float(np.percentile(lat, 50)), p99_us=float(np.percentile(lat, 99)))


def fmatrix_run(device, cfg, init, arr, steps=8, warmup=2):
    """K2 with the score matrix materialised (the c4 batch): every (waiting request, worker) pair of the
    step-start snapshot written to HBM, 4 B per pair, plus both reductions; the round follows as its own launch."""
    import torch
    from paper_2605_06113_amd import binding
    routers = [binding.Router(cfg, init, device=device) for _ in range(steps + warmup)]
    darr = binding.DeviceArrivals(arr, device, 0)
    out = routers[0].alloc_outputs(scores=False)      # the matrix alone: its kernel is timed by itself
    out["F"] = torch.zeros((cfg.n_inst, cfg.max_wait, cfg.G), dtype=torch.int32, device=device)
    for r in routers[:warmup]:
        r.route_step_device(darr, out)
    torch.cuda.synchronize()
    for r in routers[warmup:]:
        r.profile(True)       # every step: this leg reports the matrix kernel's own duration
    t0 = time.perf_counter()
    for r in routers[warmup:]:
        r.route_step_device(darr, out)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    st = out["stats"].cpu().numpy()
    qn = int(st[:, binding.ST["qlen"]].sum())
    ms = cnt = 0
    for r in routers[warmup:]:
        m, c = r.profile_read()["score"]
        ms += m
        cnt += c
    for r in routers:
        r.close()
    avg = ms / max(cnt, 1)
    N, G = cfg.n_inst, cfg.G
    nbytes = qn * G * 4 + qn * 4 + N * G * 4                # matrix written; prefill lengths and loads read
    gbs = nbytes / (avg * 1e-3) / 1e9
    return dict(workload="c4 batch, br_route_step with F requested: score matrix (4096 x 256 x 16 int32), then the round",
                kernel="br_k_score_matrix<false,false>", kernel_avg_ms=avg, launches=cnt, bytes_per_launch=nbytes, bound="hbm",
                achieved_GBs=gbs, frac=gbs / HBM_PEAK_GBS, pairs_per_s=qn * G / (avg * 1e-3),
                ms_per_round_with_matrix=elapsed / steps * 1e3)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--latency-steps", type=int, default=10000,
                    help="decode steps of the single-instance latency replay (the stress shape runs 10000)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-only", action="store_true",
                    help="print only the oracle's timing (JSON); what the default run starts as a child process, so "
                         "that the oracle's worker processes are forked from a process that never touched the GPU")
    ap.add_argument("--profile-every", type=int, default=4,
                    help="bracket the kernels of every n-th timed step with HIP events (per-kernel durations)")
    ap.add_argument("--two-calls", action="store_true",
                    help="time br_route_step + br_advance_decode instead of the fused br_route_advance")
    ap.add_argument("--no-two-calls-leg", action="store_true", help="skip the side measurement of the two-call step")
    ap.add_argument("--no-brh", action="store_true", help="skip the side legs")
    ap.add_argument("--legs", default="all",
                    help="comma-separated side legs to run (fmatrix,brh,brh_gate_off,h80,window16,window32,window32_all,bypass,"
                         "replay,quality), default all")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for scaling rocprofv3 byte counters)")
    ap.add_argument("--traffic-kib", type=float, default=None,
                    help="HBM KiB per launch of the dominant kernel from rocprofv3 --pmc runs, if known")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (instances shard across GPUs with no exchange); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.cpu_baseline_only:
        from paper_2605_06113_amd import workloads as wl
        cfg = wl.config("c4")
        print(json.dumps(cpu_baseline(cfg, wl.initial_state(cfg), wl.initial_waiting(cfg))))
        return

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

    # Algorithmic work per launch (HBM bytes the step has to move, whatever the kernel does):
    #   decode step (K5): 16 B per occupied slot (kv, rem read and written);
    #   round (K4), per instance: 4 R (prefill lengths read) + 4 R (assignments written) + 16 G (L, n read and
    #     written) + (8 + 4 H) per admission (kv, rem and prediction row of the new list entry), H = 0 here;
    #   snapshot reductions (K2 + K3) without the matrix: their outputs, 4 R + 4 G per instance (inputs are K4's).
    N, G, B, Q = cfg.n_inst, cfg.G, cfg.B, cfg.max_wait
    occupied_after = N * G * 128 + admitted          # slots the decode step touches
    bytes_advance = occupied_after * 16
    bytes_assign = qn * 4 + qn * 4 + N * G * 16 + admitted * 8
    bytes_score = qn * 4 + N * G * 4
    # side figure: integer operations of the method itself, 4 per score; every admission scores the requests still
    # waiting at that moment (qn, qn - 1, ...), the snapshot scores every pair once
    st_q = stats[:, binding.ST["qlen"]].astype(np.float64)
    st_a = stats[:, binding.ST["admitted"]].astype(np.float64)
    ops_assign = 4.0 * float((st_a * st_q - st_a * (st_a - 1) / 2).sum())
    counters = profile_counters()
    kname = {(True, "assign"): "br_k_route4<true>", (False, "assign"): "br_k_route4<false>",
             (True, "advance"): "br_k_advance<1,2,false>", (False, "advance"): "br_k_advance<1,2,false>"}

    def kernel_table(kern, fused):
        tab = {}
        for k, (ms, c) in kern.items():
            if c == 0:
                continue
            avg = ms / c
            e = dict(avg_ms=avg, launches=c)
            if k == "advance":
                nb = bytes_advance
            elif k == "score":
                nb = bytes_score + qn * 4 + N * G * 8
            elif k == "assign":
                # on this workload the snapshot reductions ride in the round's launch (br_k_route4); the fused
                # launch also applies the decode step
                nb = bytes_assign + bytes_score + (bytes_advance if fused else 0)
                ops = ops_assign + 4.0 * pairs_per_step
                e.update(alu=dict(achieved_Tops=ops / (avg * 1e-3) / 1e12, peak_Tops=ALU_INT_PEAK_TOPS,
                                  frac=ops / (avg * 1e-3) / 1e12 / ALU_INT_PEAK_TOPS,
                                  ops="4 per (admission, request still waiting) + 4 per snapshot pair"),
                         includes_snapshot_reductions=True, includes_decode_step=bool(fused))
            else:
                tab[k] = e
                continue
            gbs = nb / (avg * 1e-3) / 1e9
            e.update(bound="hbm", kernel=kname.get((bool(fused), k), k), bytes_per_launch=nb, achieved_GBs=gbs,
                     frac=gbs / HBM_PEAK_GBS)
            tab[k] = e
        return tab

    per_kernel = kernel_table(kern, fused)
    dom = max((k for k in per_kernel if k != "init"), key=lambda k: per_kernel[k]["avg_ms"])
    d = per_kernel[dom]
    roofline = dict(bound="hbm", kernel=d["kernel"], achieved=d["achieved_GBs"], peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=d["frac"], bytes_per_launch=d["bytes_per_launch"], avg_launch_ms=d["avg_ms"])
    # HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (profiles/); null once the sources changed
    tb = args.traffic_kib * 1024.0 if args.traffic_kib is not None else counters.get("traffic_bytes " + d["kernel"])
    roofline["traffic"] = tb
    if "alu" in d:
        roofline["alu"] = d["alu"]
        # LDS traffic of the round kernel: instructions per wave from rocprofv3 --pmc SQ_INSTS_LDS (profiles/), taken
        # as 64 lanes x 4 B each, against 128 B per clock and CU; the dependent chain lives in registers and DPP
        lpw = counters.get("lds_insts_per_wave " + d["kernel"])
        if lpw is not None:
            lds_gbs = lpw * 64 * 4 * cfg.n_inst / (d["avg_ms"] * 1e-3) / 1e9
            roofline["lds"] = dict(achieved_GBs=lds_gbs, peak_GBs=LDS_PEAK_GBS, frac=lds_gbs / LDS_PEAK_GBS,
                                   insts_per_wave=lpw)
        else:
            roofline["lds"] = None
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
        legs = dict(fmatrix=lambda: fmatrix_run(device, cfg, init, arr), brh=lambda: brh_run(device),
                    brh_gate_off=lambda: brh_run(device, gate=0.0),   # hazards live: no request counts at the last offset
                    h80=lambda: brh_run(device, deployed=True), window16=lambda: window_run(device),
                    window32=lambda: window_run(device, R_max=32),   # reachable sums instead of masks
                    window32_all=lambda: window_run(device, R_max=32, S_greedy=512),
                    bypass=lambda: bypass_run(device, cfg, init, arr), replay=lambda: replay_run(device),
                    quality=lambda: quality_run(device))
        keys = dict(brh="brh_batched", brh_gate_off="brh_batched_gate_off", h80="brh_batched_h80",
                    window32_all="window32_all_stage2", replay="replay_batched")
        want = list(legs) if args.legs == "all" else [x for x in args.legs.split(",") if x]
        for name in want:
            res[keys.get(name, name)] = legs[name]()
    if args.latency_steps > 0:
        res["latency"] = latency_run(args.latency_steps, device)
        res["latency_c1"] = c1_latency(device)
        res["latency_c2"] = latency_run(args.latency_steps, device, name="c2")
        res["latency_c3"] = latency_run(args.latency_steps, device, name="c3")
        res["latency_deployed"] = latency_run(min(args.latency_steps, 4000), device, deployed=True)
    if not args.no_cpu_baseline:
        import subprocess
        torch.cuda.synchronize()
        child = subprocess.run([sys.executable, os.path.abspath(__file__), "--cpu-baseline-only"], capture_output=True,
                               text=True, timeout=600)
        if child.returncode != 0:
            print(child.stderr, file=sys.stderr)
            raise RuntimeError("the oracle timing leg failed")
        res["cpu_baseline"] = json.loads(child.stdout.strip().splitlines()[-1])
    print(json.dumps(res))


if __name__ == "__main__":
    main()
