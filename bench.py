"""Benchmark of the planner-search hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic candidates, inputs resident in
HBM: build the segment-cost tables, plan every candidate (recurrence, backtrack, fused score),
select the best plan.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload stress] [--path auto|generic]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# int32 VALU peak of one MI355X: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second
ALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9
# Accounting convention for one transition (s, i, j) of the recurrence: 13 integer operations (time:
# 2 sub, add, shift, add; memory: 2 sub, mul, add, compare; combine: 2 max, 1 min-select).  On the int64
# path each is a 64-bit operation = two 32-bit lane-operations (26 per transition); on the 32-bit path,
# which the table build has proven exact for the problem, each is one lane-operation (13).
LANE_OPS_PER_TRANSITION = {"int64": 26, "u32": 13}
# sources of the planner kernel; counter-derived figures in profiles/ are quoted only while these are unchanged
KERNEL_SOURCES = ("k2_fast.hip", "fast_common.h", "plan_common.h", "harp_internal.h")
COUNTER_FILE = os.path.join(ROOT, "profiles", "plan_batch_stress_counters.json")
TABLES_COUNTER_FILE = os.path.join(ROOT, "profiles", "tables_streaming_counters.json")


def kernel_source_hash():
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2509_24859_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def counter_figures(workload, full_batch):
    """HBM traffic and the issued-instruction view of the planner launch from the rocprofv3 counter runs
    recorded in profiles/ - quoted only when they were taken on this workload with the kernel sources as
    they are now (the record carries their hash); otherwise None, never a stale number."""
    if not full_batch or not os.path.exists(COUNTER_FILE):
        return None, None
    with open(COUNTER_FILE) as f:
        rec = json.load(f)
    if rec.get("workload") != workload or rec.get("kernel_source_hash") != kernel_source_hash():
        return None, None
    return rec.get("traffic_bytes_per_call"), rec.get("issued")


def tables_traffic(L):
    """HBM traffic of one table build from the rocprofv3 counter runs recorded in profiles/, quoted only
    for the length they were taken at and while the kernel source is what it was then."""
    import hashlib
    if not os.path.exists(TABLES_COUNTER_FILE):
        return None
    with open(TABLES_COUNTER_FILE) as f:
        rec = json.load(f)
    with open(os.path.join(ROOT, "paper_2509_24859_amd", "csrc", "k1_tables.hip"), "rb") as f:
        now = hashlib.sha256(f.read()).hexdigest()[:16]
    if rec.get("L") != L or rec.get("kernel_source_hash") != now:
        return None
    return rec.get("traffic_bytes_per_build")


def cpu_baseline(w, cands, gpu_plans, budget_candidates):
    """The oracle as it stands, timed on the host cores over the first candidates of the batch;
    the same run checks the GPU's plans for those candidates bit for bit."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import oracle
    from paper_2509_24859_amd import workloads

    cores = min(16, len(os.sched_getaffinity(0)))
    n = min(cands.C, budget_candidates)
    sample = cands.slice(0, n)
    tables = oracle.build_tables(w.problem)
    out = oracle.Plans(n, sample.S_max)
    step = max(1, min(16, n // (cores * 4) or 1))
    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        list(ex.map(lambda lo: oracle.plan_batch(tables, sample, lo, min(lo + step, n), out),
                    range(0, n, step)))
    dt = time.perf_counter() - t0
    for name in ("status", "splits", "dev_first", "bottleneck", "iter_time"):
        if not (getattr(out, name) == getattr(gpu_plans, name)[:n]).all():
            raise SystemExit("GPU plans differ from the oracle in %s on the baseline sample" % name)
    cells, trans = workloads.dense_counts(w.problem.L, sample.cand_S)
    return {"value": n / dt, "unit": "plans/s", "cores": cores, "kind": "oracle",
            "sample": "first %d candidates of the %s batch, %d threads over candidates, %.1f s wall; "
                      "GPU plans for the sample verified bit-exact in the same run" % (n, w.name, cores, dt),
            "transitions_per_s": float(trans.sum()) / dt, "cells_per_s": float(cells.sum()) / dt}


def device_state():
    """Clock and power state of the first GPU as the amdgpu driver publishes it in sysfs, read
    before the run (plain file reads: no child process is started)."""
    import glob
    state = {}
    for card in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
        if not os.path.exists(os.path.join(card, "pp_dpm_sclk")):
            continue
        for name in ("pp_dpm_sclk", "pp_dpm_mclk", "power_dpm_force_performance_level"):
            try:
                with open(os.path.join(card, name)) as f:
                    lines = [x.strip() for x in f.read().strip().splitlines()]
            except OSError as e:
                state[name] = "unreadable: %s" % e.strerror
                continue
            current = [x for x in lines if x.endswith("*")]
            state[name] = {"levels": lines, "current": current[0] if current else None} if len(lines) > 1 else lines[0]
        state["card"] = card
        break
    return state or {"error": "no amdgpu clock files under /sys/class/drm"}


def tables_streaming(ctx, binding, workloads, torch, L, reps=10):
    """Table build alone on an operator-level sequence: the launch that is HBM-bound by nature but
    moves under 3 MB at the planner's own sizes.  Algorithmic bytes: every input read once, every
    table row written once."""
    p = workloads.long_sequence(L)
    tables = binding.Tables(ctx, p)
    n_rows = p.T + 2 + p.G * len(p.tp_degrees)
    bytes_alg = (2 * p.T + 3) * 8 * p.L + n_rows * 8 * (p.L + 1)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    tables.rebuild()
    torch.cuda.synchronize()
    a.record()
    for _ in range(reps):
        tables.rebuild()
    b.record()
    torch.cuda.synchronize()
    tables.finalize()
    ms = a.elapsed_time(b) / reps
    rate = bytes_alg / (ms * 1e-3)
    return {"kernel": "k1 (chunk sums, chunk-sum scan, row scan, finalize)", "L": p.L, "rows": n_rows,
            "algorithmic_bytes": bytes_alg, "ms_per_build": ms, "bound": "hbm",
            "achieved": rate / 1e9, "peak": 8000.0, "unit": "GB/s", "frac": rate / 8e12,
            "traffic": tables_traffic(p.L)}


def measured_peaks(ctx, binding, torch):
    """What this GPU sustains, measured in the same run: 32-bit integer vector operations (a kernel
    of nothing but independent add/max chains, 8 waves per SIMD) and a plain device-to-device copy."""
    sink = torch.zeros(1, dtype=torch.int32, device=ctx.device)
    blocks, iters = 256 * 8 * 4, 4096
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    binding.harp_measure_valu_int32(ctx, blocks, 64, sink)
    torch.cuda.synchronize()
    a.record()
    binding.harp_measure_valu_int32(ctx, blocks, iters, sink)
    b.record()
    torch.cuda.synchronize()
    valu = blocks * 256 * iters * 16 / (a.elapsed_time(b) * 1e-3)
    src = torch.ones(1 << 30, dtype=torch.uint8, device=ctx.device)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    a.record()
    for _ in range(4):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    copy = 4 * 2 * src.numel() / (a.elapsed_time(b) * 1e-3)
    del src, dst
    return {"valu_int32_lane_ops_per_s": valu, "valu_frac_of_nominal": valu / ALU_PEAK_LANE_OPS,
            "hbm_copy_bytes_per_s": copy, "hbm_copy_frac_of_nominal": copy / 8e12,
            "note": "add/max chains, 8192 workgroups x 256 threads x 65536 ops per lane; "
                    "1 GiB device-to-device copy, read + written bytes"}


def timed_ms(torch, fn, reps, warmup=1):
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def graph_replay(ctx, binding, torch, tables, dc, out, ws, best_t, best_i, reps):
    """plan + argmin of one step captured once in a HIP graph and replayed: what a caller that plans
    many small batches saves in launch overhead (the table build stays outside: its verdict is read
    back on the host)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())

    def body(stream):
        binding.harp_plan_batch(ctx, tables, dc, out, ws, stream)
        binding.harp_argmin_batch(ctx, dc.C, out.iter_time, out.status, best_t, best_i, stream)

    with torch.cuda.stream(side):
        body(side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        body(torch.cuda.current_stream())
    eager = timed_ms(torch, lambda: body(None), reps)
    replay = timed_ms(torch, graph.replay, reps)
    return {"eager_ms": eager, "replay_ms": replay, "launches_captured": 4}


def exact_search(ctx, binding, torch, w, tables, dc, cands, minmax, reps, cpu_candidates):
    """The exact search (cap sweep on top of the min-max plans) over the same batch: time per call,
    capped passes per candidate, what it gains over the min-max plans, and the oracle's sweep timed
    on a few candidates (which also checks the GPU's answers for them bit for bit)."""
    import numpy as np

    out = binding.DevicePlans(ctx, dc.C, dc.S_max)
    ws = binding.plan_workspace(ctx, tables, dc)
    n_passes = torch.zeros(dc.C, dtype=torch.int32, device=ctx.device)
    binding.harp_plan_exact_batch(ctx, tables, dc, out, ws, n_passes)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        binding.harp_plan_exact_batch(ctx, tables, dc, out, ws, n_passes)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / reps
    got = out.to_host()
    passes = n_passes.cpu().numpy()
    ok = got.status == 0
    gain = 1.0 - got.iter_time[ok] / np.maximum(1, minmax.iter_time[ok])
    res = {"kernel": "k2_band + k2_fast + k2_exact (one harp_plan_exact_batch call)", "ms_per_call": ms,
           "plans_per_s": dc.C / (ms * 1e-3), "capped_passes_total": int(passes.sum()),
           "capped_passes_mean_feasible": float(passes[ok].mean()) if ok.any() else 0.0,
           "capped_passes_max": int(passes.max()) if passes.size else 0,
           "improved_fraction": float((got.iter_time[ok] < minmax.iter_time[ok]).mean()) if ok.any() else 0.0,
           "mean_iter_time_gain": float(gain.mean()) if ok.any() else 0.0,
           "best_iter_time_us": int(got.iter_time[ok].min()) if ok.any() else None,
           "_caps": np.where(ok, got.bottleneck, 0).astype(np.int64)}
    if cpu_candidates:
        import oracle
        from concurrent.futures import ThreadPoolExecutor
        cores = min(16, len(os.sched_getaffinity(0)))
        idx = np.nonzero(ok)[0][:cpu_candidates]
        sub = cands.take(idx)
        ot = oracle.build_tables(w.problem)
        want = oracle.Plans(sub.C, sub.S_max)
        want.n_caps = np.zeros(sub.C, dtype=np.int32)
        t0 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            list(ex.map(lambda c: oracle.plan_exact_batch(ot, sub, c, c + 1, want), range(sub.C)))
        dt = time.perf_counter() - t0
        for name in ("status", "splits", "bottleneck", "iter_time"):
            if not (getattr(want, name) == getattr(got, name)[idx]).all():
                raise SystemExit("GPU exact plans differ from the oracle in %s on the baseline sample" % name)
        res["cpu_baseline"] = {"value": sub.C / dt, "unit": "plans/s", "cores": cores, "kind": "oracle",
                               "sample": "first %d feasible candidates of the batch, one per task over %d threads, "
                                         "%.1f s wall, %d caps swept per candidate on average; GPU answers for "
                                         "the sample verified bit-exact" % (sub.C, cores, dt, want.n_caps.mean())}
    return res


def h1f1b_search(ctx, binding, torch, w, tables, dc, cands, caps_host, reps, cpu_candidates):
    """The capped recurrence with H-1F1B warm-up counts over the same batch, every candidate under
    the cap the exact search chose for it: time per call, feasible fraction, and the oracle timed on
    the first candidates (which also checks the GPU's answers for them bit for bit)."""
    import numpy as np

    out = binding.DevicePlans(ctx, dc.C, dc.S_max)
    ws = binding.plan_workspace(ctx, tables, dc)
    caps = torch.from_numpy(np.ascontiguousarray(caps_host, dtype=np.int64)).to(ctx.device)
    warmup = torch.empty((dc.C, dc.S_max), dtype=torch.int32, device=ctx.device)
    ms = timed_ms(torch, lambda: binding.harp_plan_h1f1b_batch(ctx, tables, dc, caps, out, warmup, ws), reps)
    got = out.to_host()
    got.warmup = warmup.cpu().numpy()
    ok = got.status == 0
    res = {"kernel": "k2_band + k2_h1f1b (one harp_plan_h1f1b_batch call)", "ms_per_call": ms,
           "plans_per_s": dc.C / (ms * 1e-3), "feasible_fraction": float(ok.mean()),
           "mean_first_stage_warmup": float(got.warmup[ok, 0].mean()) if ok.any() else None,
           "caps": "bottleneck of the exact search's plan per candidate"}
    if cpu_candidates:
        import oracle
        from concurrent.futures import ThreadPoolExecutor
        cores = min(16, len(os.sched_getaffinity(0)))
        n = min(cands.C, cpu_candidates)
        sub = cands.slice(0, n)
        ot = oracle.build_tables(w.problem)
        want = oracle.Plans(n, sub.S_max)
        want.warmup = np.full((n, sub.S_max), -1, dtype=np.int32)
        sub_caps = np.ascontiguousarray(caps_host[:n], dtype=np.int64)
        t0 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            list(ex.map(lambda lo: oracle.plan_h1f1b_batch(ot, sub, sub_caps, lo, min(lo + 8, n), want),
                        range(0, n, 8)))
        dt = time.perf_counter() - t0
        for name in ("status", "splits", "dev_first", "warmup", "bottleneck", "iter_time"):
            if not (getattr(want, name) == getattr(got, name)[:n]).all():
                raise SystemExit("GPU H-1F1B plans differ from the oracle in %s on the baseline sample" % name)
        res["cpu_baseline"] = {"value": n / dt, "unit": "plans/s", "cores": cores, "kind": "oracle",
                               "sample": "first %d candidates of the batch over %d threads, %.1f s wall; GPU "
                                         "answers for the sample verified bit-exact" % (n, cores, dt)}
    return res


def mesh_search(ctx, binding, torch, workloads, name, n_orders, reps, cpu_orders, sweep_orders):
    """The planner that chooses the slicing inside the recurrence, over a batch of random group
    orderings of one of the smaller workloads (the state space has a device dimension, so the work
    per ordering is devices x degrees times that of a hot-path candidate)."""
    import numpy as np

    w = workloads.make(name)
    p = w.problem
    orders = workloads.make_orderings(p, w.seed, w.config_id, p.G, w.S_max, 0, n_orders)
    tables = binding.Tables(ctx, p)
    do = binding.DeviceOrderings(ctx, orders)
    out = binding.DevicePlans(ctx, do.C, do.S_max)
    sg = torch.empty((do.C, do.S_max), dtype=torch.int32, device=ctx.device)
    st = torch.empty_like(sg)
    ws = binding.mesh_workspace(ctx, tables, do)
    ms = timed_ms(torch, lambda: binding.harp_plan_mesh_batch(ctx, tables, do, out, sg, st, ws), reps)
    got = out.to_host()
    ok = got.status == 0
    S = orders.ord_S.astype(np.float64)
    dense = float((S * p.L * p.L / 2 * int(p.group_ndev.sum()) * len(p.tp_degrees)).sum())
    res = {"kernel": "k2_mesh (one harp_plan_mesh_batch call)", "workload": "%s: L=%d, %d devices in %d groups, %d orderings, S<=%d"
           % (name, p.L, int(p.group_ndev.sum()), p.G, do.C, do.S_max), "ms_per_call": ms,
           "orderings_per_s": do.C / (ms * 1e-3), "dense_transitions_per_s": dense / (ms * 1e-3),
           "feasible_fraction": float(ok.mean()), "workspace_bytes": int(ws.numel())}
    # the full recurrence (device index and H-1F1B count) under caps one eighth above the min-max bottleneck
    caps_host = np.where(ok, got.bottleneck // 8 * 9, -1).astype(np.int64)
    caps = torch.from_numpy(caps_host).to(ctx.device)
    out_h = binding.DevicePlans(ctx, do.C, do.S_max)
    wu = torch.empty_like(sg)
    ms_h = timed_ms(torch, lambda: binding.harp_plan_mesh_h1f1b_batch(ctx, tables, do, caps, out_h, sg, st, wu, ws), reps)
    res["h1f1b_ms_per_call"] = ms_h
    got_h = out_h.to_host()
    got_h.warmup = wu.cpu().numpy()
    res["h1f1b_feasible_fraction"] = float((got_h.status == 0).mean())
    # the exact form: the capped least-sum pass walked over the caps
    npass = torch.empty(do.C, dtype=torch.int32, device=ctx.device)
    out_e = binding.DevicePlans(ctx, do.C, do.S_max)
    ms_e = timed_ms(torch, lambda: binding.harp_plan_mesh_exact_batch(ctx, tables, do, out_e, sg, st, ws, npass), reps)
    got_e = out_e.to_host()
    res["exact_ms_per_call"] = ms_e
    res["exact_mean_capped_passes"] = float(npass.cpu().numpy()[ok].mean()) if ok.any() else None
    res["exact_mean_gain_over_min_max"] = (float((1.0 - got_e.iter_time[ok] / got.iter_time[ok]).mean())
                                           if ok.any() else None)
    # the search around the full recurrence: every candidate cap from t_S to ceil(T / B), one pass each
    n_sweep = min(do.C, sweep_orders)
    if n_sweep:
        sub = orders.slice(0, n_sweep)
        ds = binding.DeviceOrderings(ctx, sub)
        out_s = binding.DevicePlans(ctx, ds.C, ds.S_max)
        tm = torch.empty(ds.C, dtype=torch.int64, device=ctx.device)
        nc = torch.empty(ds.C, dtype=torch.int32, device=ctx.device)
        ws_s = binding.mesh_sweep_workspace(ctx, tables, ds)
        sg_s, st_s, wu_s = (torch.empty((ds.C, ds.S_max), dtype=torch.int32, device=ctx.device) for _ in range(3))
        run = lambda cap_limit: binding.harp_plan_mesh_h1f1b_sweep_batch(ctx, tables, ds, cap_limit, out_s, sg_s, st_s,
                                                                         wu_s, tm, ws_s, nc)
        ms_s = timed_ms(torch, lambda: run(1 << 20), 1, warmup=0)
        got_s = out_s.to_host()
        oks = got_s.status == 0
        tried = nc.cpu().numpy()
        res["sweep"] = {"kernel": "k2_mesh_h1f1b_sweep (one harp_plan_mesh_h1f1b_sweep_batch call)",
                        "orderings": int(ds.C), "ms_per_call": ms_s, "mean_caps_tried": float(tried.mean()),
                        "max_caps_tried": int(tried.max()), "passes_per_s": float(tried.sum()) / (ms_s * 1e-3),
                        "feasible_fraction": float(oks.mean())}
        if cpu_orders:
            import oracle
            from concurrent.futures import ThreadPoolExecutor
            # the oracle under a limit of 24 caps on the first orderings, the GPU under the same limit
            n_chk, limit = min(ds.C, 16), 24
            run(limit)
            torch.cuda.synchronize()
            lim = out_s.to_host()
            ot = oracle.build_tables(p)
            want = None
            t0 = time.perf_counter()
            with ThreadPoolExecutor(min(16, len(os.sched_getaffinity(0)))) as ex:
                outs = list(ex.map(lambda c: oracle.plan_mesh_h1f1b_sweep_batch(ot, sub, limit, c, c + 1), range(n_chk)))
            dt = time.perf_counter() - t0
            for c, want in enumerate(outs):
                for name in ("status", "splits", "dev_first", "bottleneck", "iter_time"):
                    if not (getattr(want, name)[c] == getattr(lim, name)[c]).all():
                        raise SystemExit("GPU sweep differs from the oracle in %s at ordering %d" % (name, c))
                if want.t_max[c] != int(tm[c].item()) or want.n_caps[c] != int(nc[c].item()):
                    raise SystemExit("GPU sweep differs from the oracle in the cap chosen at ordering %d" % c)
            res["sweep"]["cpu_baseline"] = {"value": n_chk * limit / dt, "unit": "capped passes/s", "cores": min(16, len(os.sched_getaffinity(0))),
                                            "kind": "oracle", "sample": "first %d orderings under a limit of %d caps, "
                                            "one ordering per thread, %.1f s wall; GPU answers under the same limit "
                                            "verified bit-exact" % (n_chk, limit, dt)}
    # the same search for candidates of this workload (fixed slicing)
    if sweep_orders:
        cands = w.candidates(0, min(w.C, sweep_orders))
        dcs = binding.DeviceCandidates(ctx, cands)
        out_c = binding.DevicePlans(ctx, dcs.C, dcs.S_max)
        wu_c = torch.empty((dcs.C, dcs.S_max), dtype=torch.int32, device=ctx.device)
        tm_c = torch.empty(dcs.C, dtype=torch.int64, device=ctx.device)
        nc_c = torch.empty(dcs.C, dtype=torch.int32, device=ctx.device)
        ws_c = binding.h1f1b_sweep_workspace(ctx, tables, dcs)
        ms_c = timed_ms(torch, lambda: binding.harp_plan_h1f1b_sweep_batch(ctx, tables, dcs, 1 << 20, out_c, wu_c, tm_c,
                                                                           ws_c, nc_c), 1, warmup=0)
        tried_c = nc_c.cpu().numpy()
        res["candidate_sweep"] = {"kernel": "k2_mesh_h1f1b_sweep, fixed slicing (one harp_plan_h1f1b_sweep_batch call)",
                                  "candidates": int(dcs.C), "ms_per_call": ms_c,
                                  "mean_caps_tried": float(tried_c.mean()), "max_caps_tried": int(tried_c.max()),
                                  "passes_per_s": float(tried_c.sum()) / (ms_c * 1e-3),
                                  "feasible_fraction": float((out_c.to_host().status == 0).mean())}
        if cpu_orders:
            import oracle
            from concurrent.futures import ThreadPoolExecutor
            n_chk, limit = min(dcs.C, 16), 24
            binding.harp_plan_h1f1b_sweep_batch(ctx, tables, dcs, limit, out_c, wu_c, tm_c, ws_c, nc_c)
            torch.cuda.synchronize()
            lim = out_c.to_host()
            ot = oracle.build_tables(p)
            with ThreadPoolExecutor(min(16, len(os.sched_getaffinity(0)))) as ex:
                outs = list(ex.map(lambda c: oracle.plan_h1f1b_sweep_batch(ot, cands, limit, c, c + 1), range(n_chk)))
            for c, want in enumerate(outs):
                for name in ("status", "splits", "dev_first", "bottleneck", "iter_time"):
                    if not (getattr(want, name)[c] == getattr(lim, name)[c]).all():
                        raise SystemExit("GPU candidate sweep differs from the oracle in %s at candidate %d" % (name, c))
                if want.t_max[c] != int(tm_c[c].item()) or want.n_caps[c] != int(nc_c[c].item()):
                    raise SystemExit("GPU candidate sweep differs from the oracle in the cap chosen at candidate %d" % c)
            res["candidate_sweep"]["check"] = ("first %d candidates under a limit of %d caps verified bit-exact "
                                               "against the oracle" % (n_chk, limit))
    timed_ms(torch, lambda: binding.harp_plan_mesh_batch(ctx, tables, do, out, sg, st, ws), 1)   # restore sg, st
    if cpu_orders:
        import oracle
        from concurrent.futures import ThreadPoolExecutor
        cores = min(16, len(os.sched_getaffinity(0)))
        n = min(do.C, cpu_orders)
        sub = orders.slice(0, n)
        ot = oracle.build_tables(p)
        want = oracle.Plans(n, sub.S_max)
        want.stage_group = np.full((n, sub.S_max), -1, dtype=np.int32)
        want.stage_tp = np.full((n, sub.S_max), -1, dtype=np.int32)
        t0 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            list(ex.map(lambda c: oracle.plan_mesh_batch(ot, sub, c, c + 1, want), range(n)))
        dt = time.perf_counter() - t0
        for field in ("status", "splits", "dev_first", "bottleneck", "iter_time"):
            if not (getattr(want, field) == getattr(got, field)[:n]).all():
                raise SystemExit("GPU submesh plans differ from the oracle in %s on the baseline sample" % field)
        if not (want.stage_tp == st[:n].cpu().numpy()).all() or not (want.stage_group == sg[:n].cpu().numpy()).all():
            raise SystemExit("GPU submesh slicings differ from the oracle on the baseline sample")
        # the H-1F1B form and the exact form of the same launches, on shorter prefixes (their oracles are slower)
        n_h, n_e = min(n, 64), min(n, 16)
        want_h = oracle.Plans(n_h, sub.S_max)
        want_h.stage_group = np.full((n_h, sub.S_max), -1, dtype=np.int32)
        want_h.stage_tp = np.full((n_h, sub.S_max), -1, dtype=np.int32)
        want_h.warmup = np.full((n_h, sub.S_max), -1, dtype=np.int32)
        sub_h, sub_e = orders.slice(0, n_h), orders.slice(0, n_e)
        want_e = oracle.Plans(n_e, sub.S_max)
        want_e.stage_group = np.full((n_e, sub.S_max), -1, dtype=np.int32)
        want_e.stage_tp = np.full((n_e, sub.S_max), -1, dtype=np.int32)
        want_e.n_caps = np.zeros(n_e, dtype=np.int32)
        t1 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            list(ex.map(lambda c: oracle.plan_mesh_h1f1b_batch(ot, sub_h, caps_host[:n_h], c, c + 1, want_h), range(n_h)))
            list(ex.map(lambda c: oracle.plan_mesh_batch(ot, sub_e, c, c + 1, want_e, True), range(n_e)))
        dt1 = time.perf_counter() - t1
        for field in ("status", "splits", "dev_first", "bottleneck", "iter_time"):
            if not (getattr(want_h, field) == getattr(got_h, field)[:n_h]).all():
                raise SystemExit("GPU submesh H-1F1B plans differ from the oracle in %s on the baseline sample" % field)
            if not (getattr(want_e, field) == getattr(got_e, field)[:n_e]).all():
                raise SystemExit("GPU submesh exact plans differ from the oracle in %s on the baseline sample" % field)
        if not (want_h.warmup == got_h.warmup[:n_h]).all():
            raise SystemExit("GPU submesh H-1F1B counts differ from the oracle on the baseline sample")
        res["cpu_baseline"] = {"value": n / dt, "unit": "orderings/s", "cores": cores, "kind": "oracle",
                               "sample": "first %d orderings over %d threads, %.1f s wall; GPU answers for the "
                                         "sample verified bit-exact; also the H-1F1B form on the first %d and "
                                         "the exact form on the first %d (%.1f s wall, %d caps swept per "
                                         "ordering on average)" % (n, cores, dt, n_h, n_e, dt1, want_e.n_caps.mean())}
    return res


def minmax_config(ctx, binding, torch, workloads, name, reps, with_cpu):
    """One workload through the min-max path on its own: time per harp_plan_batch, rates by the fixed
    formulas of the dense recurrence, the work the kernel actually did (counted by the instrumented
    build of the same kernel), and the oracle beside it: single-thread rate on the first min(C, 1024)
    candidates, then every host thread over the whole batch, which also verifies every plan bit for bit
    (the stress batch is verified on a prefix here; the GPU test suite covers all of it)."""
    import numpy as np

    w = workloads.make(name)
    cands = w.candidates()
    cells, trans = workloads.dense_counts(w.problem.L, cands.cand_S)
    tables = binding.Tables(ctx, w.problem)
    dc = binding.DeviceCandidates(ctx, cands)
    out = binding.DevicePlans(ctx, dc.C, dc.S_max)
    ws = binding.plan_workspace(ctx, tables, dc)
    ms = timed_ms(torch, lambda: binding.harp_plan_batch(ctx, tables, dc, out, ws), reps, warmup=2)
    got = out.to_host()
    res = {"L": w.problem.L, "candidates": dc.C, "S_max": dc.S_max, "plan_kernel_ms": ms,
           "plans_per_s": dc.C / (ms * 1e-3), "cells_per_s": float(cells.sum()) / (ms * 1e-3),
           "dense_transitions_per_s": float(trans.sum()) / (ms * 1e-3),
           "feasible_fraction": float((got.status == 0).mean()), "path": "u32" if tables.fast32 else "int64"}
    if tables.fast32:
        work = torch.zeros(4, dtype=torch.int64, device=ctx.device)
        binding.harp_plan_batch_count_work(ctx, tables, dc, out, ws, work)
        torch.cuda.synchronize()
        ev, cl, tr, nc = (int(x) for x in work.cpu().numpy())
        res["evaluated"] = {"transitions": ev, "cells": cl, "groups_of_four": tr, "candidates_planned": nc}
        res["alu_frac"] = ev * LANE_OPS_PER_TRANSITION["u32"] / (ms * 1e-3) / ALU_PEAK_LANE_OPS
    if with_cpu:
        import oracle
        from concurrent.futures import ThreadPoolExecutor
        cores = min(16, len(os.sched_getaffinity(0)))
        ot = oracle.build_tables(w.problem)
        n1 = min(dc.C, 1024)
        one = oracle.Plans(n1, cands.S_max)
        sub = cands.slice(0, n1)
        t0 = time.perf_counter()
        oracle.plan_batch(ot, sub, 0, n1, one)
        dt1 = time.perf_counter() - t0
        # all host threads: the whole batch when that is a few seconds of work, else a prefix
        n_all = dc.C if float(trans.sum()) < 4e10 else max(n1, int(dc.C * 4e10 / float(trans.sum())))
        allc = cands.slice(0, n_all)
        want = oracle.Plans(n_all, cands.S_max)
        step = max(1, min(16, n_all // (cores * 4) or 1))
        t0 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            list(ex.map(lambda lo: oracle.plan_batch(ot, allc, lo, min(lo + step, n_all), want), range(0, n_all, step)))
        dta = time.perf_counter() - t0
        for field in ("status", "splits", "dev_first", "bottleneck", "iter_time"):
            if not (getattr(want, field) == getattr(got, field)[:n_all]).all():
                raise SystemExit("GPU plans differ from the oracle in %s on workload %s" % (field, name))
        res["cpu_baseline"] = {
            "kind": "oracle", "single_thread_transitions_per_s": float(trans[:n1].sum()) / dt1,
            "single_thread_sample": "first %d candidates, %.2f s" % (n1, dt1),
            "all_core_plans_per_s": n_all / dta, "all_core_transitions_per_s": float(trans[:n_all].sum()) / dta,
            "cores": cores, "all_core_sample": "%d of %d candidates, %.2f s wall" % (n_all, dc.C, dta),
            "verified": "GPU plans of those %d candidates bit-exact against the oracle" % n_all}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="stress")
    ap.add_argument("--path", default="auto", choices=("auto", "generic", "fast32"))
    ap.add_argument("--candidates", type=int, default=0, help="use only the first N candidates")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the VALU and copy micro-benchmarks")
    ap.add_argument("--no-configs", action="store_true", help="skip the per-workload table (all five configs)")
    ap.add_argument("--cpu-candidates", type=int, default=0)
    ap.add_argument("--tables-L", type=int, default=1 << 20,
                    help="operators of the table-build streaming measurement (0 = skip)")
    ap.add_argument("--graph-reps", type=int, default=20,
                    help="replays of plan + argmin captured in a HIP graph (0 = skip)")
    ap.add_argument("--exact-reps", type=int, default=3,
                    help="timed calls of the exact search over the same batch (0 = skip)")
    ap.add_argument("--exact-cpu-candidates", type=int, default=16)
    ap.add_argument("--h1f1b-reps", type=int, default=3,
                    help="timed calls of the H-1F1B recurrence at the exact search's caps (0 = skip)")
    ap.add_argument("--h1f1b-cpu-candidates", type=int, default=1024)
    ap.add_argument("--h1f1b-workload", default="finegrained",
                    help="second workload for the H-1F1B recurrence, one where most candidates stay feasible ('' = skip)")
    ap.add_argument("--mesh-workload", default="llama70b")
    ap.add_argument("--mesh-orderings", type=int, default=4096,
                    help="group orderings for the submesh-in-recurrence planner (0 = skip)")
    ap.add_argument("--mesh-cpu-orderings", type=int, default=128)
    ap.add_argument("--mesh-sweep-orderings", type=int, default=256,
                    help="orderings given to the search around the full recurrence (0 = skip)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also run one plain device copy of this many MiB (reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU: this build has no multi-GPU path "
                         "(candidates would shard across GPUs with one 16-byte reduction); run with --gpus 1")

    state_before = device_state()
    import numpy as np
    import torch

    from paper_2509_24859_amd import binding, workloads

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs the GPU: there is no CPU path")
    ctx = binding.Context(0)
    props = torch.cuda.get_device_properties(0)
    w = workloads.make(args.workload)
    C = args.candidates or w.C
    cands = w.candidates(0, C)
    cells, trans = workloads.dense_counts(w.problem.L, cands.cand_S)
    n_cells, n_trans = float(cells.sum()), float(trans.sum())

    dp = binding.DeviceProblem(ctx, w.problem)
    dc = binding.DeviceCandidates(ctx, cands)
    out = binding.DevicePlans(ctx, dc.C, dc.S_max)
    tables = binding.Tables(ctx, dp)
    ws = binding.plan_workspace(ctx, tables, dc)
    best_t = torch.empty(1, dtype=torch.int64, device=ctx.device)
    best_i = torch.empty(1, dtype=torch.int32, device=ctx.device)
    path = {"auto": binding.PATH_AUTO, "generic": binding.PATH_GENERIC, "fast32": binding.PATH_FAST32}[args.path]
    ctx.set_plan_path(path)
    fast = tables.fast32 and path != binding.PATH_GENERIC
    kernel = ("k2_band + k2_fast (one harp_plan_batch call)" if fast
              else "k2_band + k2_banded (int64; k2_generic when the feasibility index does not fit)")
    width = "u32" if fast else "int64"

    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]

    def step(k=None):
        tables.rebuild()                       # a1: tables (enqueue)
        tables.finalize()                      #     verdict on the problem's values
        if k is not None:
            ev[k][0].record()
        binding.harp_plan_batch(ctx, tables, dc, out, ws)          # a2-a4
        if k is not None:
            ev[k][1].record()
        binding.harp_argmin_batch(ctx, dc.C, out.iter_time, out.status, best_t, best_i)  # a5

    if args.copy_calibration:
        src = torch.ones(args.copy_calibration << 20, dtype=torch.uint8, device=ctx.device)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(k)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    per_step = sorted(a.elapsed_time(b) for a, b in ev)
    kernel_ms = sum(per_step) / args.steps
    got = out.to_host()
    # the work the planner launch actually does, counted once by the instrumented build of the same kernel
    evaluated = None
    if fast:
        work = torch.zeros(4, dtype=torch.int64, device=ctx.device)
        check = binding.DevicePlans(ctx, dc.C, dc.S_max)
        binding.harp_plan_batch_count_work(ctx, tables, dc, check, ws, work)
        torch.cuda.synchronize()
        same = check.to_host()
        for field in ("status", "splits", "dev_first", "bottleneck", "iter_time"):
            if not (getattr(same, field) == getattr(got, field)).all():
                raise SystemExit("the counting build of the planner kernel gives different plans (%s)" % field)
        n_ev, n_cl, n_tr, n_pl = (int(x) for x in work.cpu().numpy())
        evaluated = {"transitions": n_ev, "cells": n_cl, "groups_of_four": n_tr, "candidates_planned": n_pl,
                     "fraction_of_dense_transitions": n_ev / n_trans, "fraction_of_dense_cells": n_cl / n_cells}
        del check
    # the other kernels of a step, each on its own (enqueue to enqueue, HIP events)
    parts = {"tables_build_ms": timed_ms(torch, tables.rebuild, 20),
             "argmin_ms": timed_ms(torch, lambda: binding.harp_argmin_batch(ctx, dc.C, out.iter_time, out.status,
                                                                            best_t, best_i), 20)}
    tables.finalize()
    b2 = torch.empty(dc.C, dtype=torch.int64, device=ctx.device)
    t2 = torch.empty_like(b2)
    s2 = torch.empty(dc.C, dtype=torch.int32, device=ctx.device)
    parts["score_ms"] = timed_ms(torch, lambda: binding.harp_score_1f1b(ctx, tables, dc, out.splits, b2, t2, s2), 10)
    del b2, t2, s2
    ops = LANE_OPS_PER_TRANSITION[width]
    dense_rate = n_trans * 26 / (kernel_ms * 1e-3)
    traffic, issued = counter_figures(args.workload, C == w.C and fast)
    if evaluated is not None:
        achieved = evaluated["transitions"] * ops / (kernel_ms * 1e-3)
        note = ("achieved = transitions the kernel evaluated in one launch (counted by the instrumented build of the "
                "same kernel, harp_plan_batch_count_work) x %d lane-ops / mean time of one harp_plan_batch (HIP events "
                "on the launch stream); %d = the 13 operations of a transition, each one 32-bit lane-op on this path "
                "(26 when they are 64-bit).  dense_equivalent_rate prices every transition of the dense recurrence, "
                "most of which the bands and bounded scans never evaluate: work delivered, not a fraction of anything"
                % (ops, ops))
    else:
        achieved = dense_rate
        note = ("int64 path: no evaluated-transition count; achieved = dense-recurrence transitions x 26 lane-ops / "
                "mean kernel time, an upper figure (the monotone stops skip part of them)")
    result = {
        "metric": "candidate plans/sec (and DP cells/sec) on 1 MI355X",
        "value": C * args.steps / elapsed,
        "unit": "plans/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32 times / int64 bytes" if fast else "int64",
        "data": "synthetic",
        "config": {"workload": "%s: L=%d operators, %d candidates, S<=%d, M=%d, %d groups, %d GPU types"
                               % (w.name, w.problem.L, C, w.S_max, w.problem.M, w.problem.G, w.problem.T),
                   "plan_path": args.path, "kernel": kernel},
        "cells_per_s": n_cells * args.steps / elapsed,
        "dense_transitions_per_s": n_trans * args.steps / elapsed,
        "plan_kernel_ms": kernel_ms,
        "plan_kernel_ms_median": per_step[len(per_step) // 2],
        "plan_kernel_ms_min": per_step[0],
        "other_kernels": parts,
        "feasible_fraction": float((got.status == 0).mean()),
        "best_plan": {"index": int(best_i.item()), "iter_time_us": int(best_t.item())},
        "device": {"name": props.name, "compute_units": props.multi_processor_count,
                   "max_clock_mhz": (getattr(props, "clock_rate", 0) or 0) / 1e3 or None,
                   "hbm_bytes": props.total_memory,
                   "sysfs_before_run": state_before},
        "roofline": {
            "bound": "alu", "kernel": kernel,
            "achieved": achieved / 1e12, "peak": ALU_PEAK_LANE_OPS / 1e12, "unit": "T int32 lane-op/s",
            "frac": achieved / ALU_PEAK_LANE_OPS, "traffic": traffic,
            "lane_ops_per_transition": ops, "evaluated": evaluated,
            "dense_equivalent_rate": dense_rate / 1e12,
            "issued": issued,
            "counters_from": (os.path.relpath(COUNTER_FILE, ROOT) if traffic is not None or issued is not None else None),
            "note": note,
        },
    }
    if evaluated is not None:
        result["roofline"]["evaluated_x26_over_peak"] = evaluated["transitions"] * 26 / (kernel_ms * 1e-3) / ALU_PEAK_LANE_OPS
    if not args.no_peaks:
        peaks = measured_peaks(ctx, binding, torch)
        result["measured_peaks"] = peaks
        result["roofline"]["frac_of_measured_peak"] = achieved / peaks["valu_int32_lane_ops_per_s"]
        # clock under load, read off the add/max chain: one lane-op per lane per cycle
        result["device"]["valu_clock_under_load_ghz"] = (peaks["valu_int32_lane_ops_per_s"]
                                                         / (props.multi_processor_count * 64) / 1e9)
    if args.tables_L:
        result["tables_streaming"] = tables_streaming(ctx, binding, workloads, torch, args.tables_L)
    if args.graph_reps and fast:
        result["graph_replay"] = graph_replay(ctx, binding, torch, tables, dc, out, ws, best_t, best_i, args.graph_reps)
    if args.exact_reps and fast:
        result["exact_search"] = exact_search(ctx, binding, torch, w, tables, dc, cands, got, args.exact_reps,
                                              0 if args.no_cpu_baseline else args.exact_cpu_candidates)
        result["_exact_caps"] = result["exact_search"].pop("_caps")
    if args.h1f1b_reps and fast and "exact_search" in result:
        result["h1f1b"] = h1f1b_search(ctx, binding, torch, w, tables, dc, cands, result.pop("_exact_caps"),
                                       args.h1f1b_reps, 0 if args.no_cpu_baseline else args.h1f1b_cpu_candidates)
    result.pop("_exact_caps", None)
    if args.h1f1b_reps and args.exact_reps and args.h1f1b_workload and args.h1f1b_workload != args.workload:
        # the same recurrence where most candidates stay feasible under H-1F1B's counts
        w2 = workloads.make(args.h1f1b_workload)
        c2 = w2.candidates()
        t2 = binding.Tables(ctx, w2.problem)
        if t2.fast32:
            d2 = binding.DeviceCandidates(ctx, c2)
            o2 = binding.DevicePlans(ctx, d2.C, d2.S_max)
            binding.harp_plan_batch(ctx, t2, d2, o2, binding.plan_workspace(ctx, t2, d2))
            torch.cuda.synchronize()
            e2 = exact_search(ctx, binding, torch, w2, t2, d2, c2, o2.to_host(), 1, 0)
            leg = h1f1b_search(ctx, binding, torch, w2, t2, d2, c2, e2.pop("_caps"), args.h1f1b_reps,
                               0 if args.no_cpu_baseline else args.h1f1b_cpu_candidates)
            leg["workload"] = "%s: L=%d, %d candidates" % (w2.name, w2.problem.L, d2.C)
            result["h1f1b_feasible_workload"] = leg
    if args.mesh_orderings:
        result["mesh"] = mesh_search(ctx, binding, torch, workloads, args.mesh_workload, args.mesh_orderings, 2,
                                     0 if args.no_cpu_baseline else args.mesh_cpu_orderings, args.mesh_sweep_orderings)
    if not args.no_configs:
        # all five workloads through the min-max path, the oracle beside each
        result["configs"] = {name: minmax_config(ctx, binding, torch, workloads, name, 20 if name != "stress" else 5,
                                                 not args.no_cpu_baseline) for name in workloads.ORDER}
    if not args.no_cpu_baseline:
        # about 20 core-seconds of oracle work at 1-5 ns per dense transition
        budget = args.cpu_candidates or max(64, int(1.6e10 / max(1.0, n_trans / C)))
        result["cpu_baseline"] = cpu_baseline(w, cands, got, budget)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
