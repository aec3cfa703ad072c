#!/usr/bin/env python3
"""Benchmark of the fused multi-tenant convolution launch on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--no-sweep] [--no-cpu]

A step is one pass of the hot path over one batch of synthetic input: every tenant's layer (or, for
configuration 5, every tenant's 53-layer stack) executed through cached plans, inputs resident in HBM.
Prints ONE JSON line.  `value` is aggregate conv TFLOP/s of the fused (space-time) policy on the
headline workload, in its fastest form: one launch sequence on one stream (`policies.fused`), or two or
four independent batches in flight on as many streams, each launch planned for its share of the GPU
(`policies.fused_pipelined`, `fused_pipelined4`; launches on one stream pay about 3 us of serialisation
each that launches on different streams overlap).  `policies` and
`per_config` carry every form of the time-only and space-only baselines (the fused plan's tiles or each
tenant planned alone; streams joined every step or free-running) and the other configurations; speed-ups
are best form against best form, `speedup_single_batch` one batch at a time.  `roofline` is measured
with HIP events on the launch stream of the single-stream form; `cpu_baseline` is the fp64 oracle timed
on this host.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6     # MI355X dense bf16/fp16 MFMA
PEAK_F32_TFLOPS = 157.3       # MI355X fp32 matrix
PEAK_HBM_GBS = 8000.0
# forms of the fused policy with several independent batches in flight: (depth of the st_pipeline, workgroup slots
# the planner fills per launch when that many launches share the GPU = st_pipeline_slots(depth))
PIPELINED = {"fused_pipelined": (2, 256), "fused_pipelined4": (4, 128)}
PAPER_CONTEXT = {"space_time_over_space_only_geomean": 3.23, "space_time_over_time_only_geomean": [7.73, 7.71],
                 "hardware": "NVIDIA V100 (AWS p3), fp32 SGEMM M=256 N=128 K=1152, 2<=R<=120",
                 "note": "other hardware and precision; context only"}

CONFIG_TEXT = {
    1: "configs[0]: 2 tenants, 3x3 s1 p1 32->32 @28x28, batch 1, fp32",
    2: "configs[1]: 4 tenants, batch 1, bf16 in / fp32 acc, ResNet-50-shaped 3x3 convs 64@56, 128@28, 256@14, 512@7",
    3: "configs[2]: 8 tenants, 3x3 256->256 @14x14, batch in {1,2,4}, bf16 in / fp32 acc",
    4: "configs[3]: 16 heterogeneous tenants (1x1, 3x3, 7x7 s2), batch 1..8, bf16 in / fp32 acc",
    5: "configs[4]: 8 tenants x 53-layer ResNet-50-shaped conv stack, batch 1, bf16, ReLU between layers",
}


def build_workload(cfg: int, copies: int = 1):
    """Returns (runner, flops, bytes, n_launches_fused, meta).  runner(policy, stream) issues one step.
    With copies > 1 (configurations 1-4) the tensors exist that many times and the "fused_cold" policy rotates
    through them, so that a launch finds none of its operands in the caches."""
    import torch
    from paper_1901_00041_amd import st_conv as sc
    from paper_1901_00041_amd import synth
    if cfg == 5:
        from paper_1901_00041_amd.stack import ResNetStack
        stack = ResNetStack(n_tenants=synth.N_TENANTS[5], cfg=5)
        twins, pipes, turn5 = {}, {}, {}

        def run5(policy: str, stream):
            if policy not in PIPELINED:
                return stack.run(policy, stream)
            # several independent batches in flight: passes rotate over as many stacks (own activations, own weights),
            # each on its own stream and planned for its share of the GPU
            depth, slots = PIPELINED[policy]
            if policy not in twins:
                twins[policy] = [ResNetStack(n_tenants=synth.N_TENANTS[5], cfg=5, seeded_weights=False,
                                             plan_opts=sc.plan_opts(target_items=slots))
                                 for _ in range(depth)]
                pipes[policy] = sc.Pipeline(depth)
                turn5[policy] = 0
            i = turn5[policy] = (turn5[policy] + 1) % depth
            twins[policy][i].run("fused", pipes[policy].next())

        def new_streams5(policy):
            if policy in pipes:
                pipes[policy] = sc.Pipeline(pipes[policy].depth)

        return run5, stack.flops, stack.bytes, stack.n_launches, {"plan_build_us": stack.plan_build_us, "pipelined": sorted(PIPELINED),
                                                                       "new_streams": new_streams5,
                                                                       "n_items": stack.n_items, "keep": stack,
                                                                       "retuned": True, "chains": True}
    dt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
    shapes = synth.config_shapes(cfg)
    keep, descs = [], []
    for t, s in enumerate(shapes):
        x = torch.from_numpy(synth.gen_input(cfg, t, 0, s).transpose(0, 2, 3, 1).copy()).to(dt[s.dtype]).cuda()
        w = torch.from_numpy(synth.gen_weight(cfg, t, 0, s).transpose(0, 2, 3, 1).copy()).to(dt[s.dtype]).cuda()
        y = torch.empty((s.N, s.P, s.Q, s.K), dtype=dt[s.out_dtype], device="cuda")
        keep.append((x, w, y))
        descs.append(sc.make_desc(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, s.dtype, s.out_dtype, x, w, y))
    t_plan = []
    for _ in range(5):
        t0 = time.perf_counter()
        plan = sc.st_conv_plan(descs, keep=keep)
        t_plan.append((time.perf_counter() - t0) * 1e6)
    info = sc.st_conv_plan_info(plan)
    streams = [torch.cuda.Stream() for _ in shapes]
    solo = [sc.st_conv_plan([d], keep=keep) for d in descs]      # each tenant planned alone (retuned baselines)
    cold_plans, cold_descs, pipe_plans, pipe_streams, pipe_turn, turn = [], [descs], {}, {}, {}, [0]
    for _ in range(copies - 1):
        cd = []
        for (x, w, y), s in zip(keep[:len(shapes)], shapes):
            x2, w2, y2 = x.clone(), w.clone(), torch.empty_like(y)
            keep.append((x2, w2, y2))
            cd.append(sc.make_desc(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, s.dtype, s.out_dtype, x2, w2, y2))
        cold_plans.append(sc.st_conv_plan(cd, keep=keep))
        cold_descs.append(cd)
    for name, (depth, slots) in PIPELINED.items():
        if copies >= depth:
            # that many launches in flight, each on its own tensors and planned for its share of the GPU
            pipe_streams[name] = sc.Pipeline(depth)
            share = sc.plan_opts(target_items=pipe_streams[name].slots)
            pipe_plans[name] = [sc.st_conv_plan(cold_descs[i], share, keep=keep) for i in range(depth)]
            pipe_turn[name] = 0

    def run(policy: str, stream):
        if policy == "fused":
            sc.st_conv_run(plan, stream)
        elif policy in PIPELINED:
            i = pipe_turn[policy] = (pipe_turn[policy] + 1) % len(pipe_plans[policy])
            pipe_streams[policy].run(pipe_plans[policy][i])
        elif policy == "fused_cold":
            turn[0] = (turn[0] + 1) % (len(cold_plans) + 1)
            sc.st_conv_run(cold_plans[turn[0] - 1] if turn[0] else plan, stream)
        elif policy == "time_only":
            sc.st_conv_run_time_only(plan, stream)
        elif policy == "space_only":
            sc.st_conv_run_space_only(plan, [stream] + streams[1:])
        elif policy == "time_only_retuned":
            sc.st_conv_run_plans_time_only(solo, stream)
        else:
            sc.st_conv_run_plans_space_only(solo, [stream] + streams[1:])

    def new_streams(policy):
        if policy in pipe_streams:
            pipe_streams[policy] = sc.Pipeline(pipe_streams[policy].depth)

    return run, int(info.flops), int(info.bytes), 1, {"plan_build_us": statistics.median(t_plan), "new_streams": new_streams,
                                                      "n_items": int(info.n_items), "keep": (plan, keep, streams, solo, cold_plans, pipe_plans, pipe_streams),
                                                      "retuned": True, "copies": copies, "pipelined": sorted(pipe_plans)}


def policy_text(form: str) -> str:
    if form in PIPELINED:
        return ("fused space-time launch, cached plans, %d independent batches in flight on as many streams, "
                "each launch planned for %d workgroup slots" % PIPELINED[form])
    if form == "fused_groups2":
        return "fused space-time launches, cached plans, two tenant groups side by side on two streams"
    return "fused space-time launch, cached plan"


def time_policy(run, policy: str, steps: int, warmup: int):
    """Wall clock (sync on both sides) and HIP-event time over exactly `steps` steps on one stream."""
    import torch
    stream = torch.cuda.Stream()
    for _ in range(warmup):
        run(policy, stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        e0.record(stream)
        for _ in range(steps):
            run(policy, stream)
        e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return wall_ms / steps, e0.elapsed_time(e1) / steps


def time_pipelined_native(pipe_plans, steps: int, warmup: int, tries: int = 3) -> float:
    """ms per step of exactly `steps` fused launches queued round-robin over len(pipe_plans) streams by the library's own
    issue loop (st_pipeline_run_many: no interpreter between launches, several issuing threads); best of `tries` freshly
    created sets of streams."""
    from paper_1901_00041_amd import st_conv as sc
    depth = len(pipe_plans)
    best = float("inf")
    for _ in range(tries):
        pipe = sc.Pipeline(depth)
        pipe.run_many(pipe_plans, max(1, warmup // depth))
        pipe.sync()
        t0 = time.perf_counter()
        pipe.run_many(pipe_plans, steps // depth)
        for i in range(steps % depth):
            pipe.run(pipe_plans[i])
        pipe.sync()
        best = min(best, (time.perf_counter() - t0) * 1e3 / steps)
        pipe.destroy()
    return best


def time_free_running(plans, streams, steps: int, warmup: int):
    """Space-only without per-step joins: plan t is launched `steps` times back to back on stream t (round-robin issue
    over the streams), the streams fork from streams[0] once before the first launch and join it once after the
    last.  Returns ms per step (one launch of every plan)."""
    import torch
    from paper_1901_00041_amd import st_conv as sc
    n = len(plans)
    use = streams[:n]
    sc.st_conv_run_plans_on_streams_many(plans, use, warmup)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record(use[0])
    for s in use[1:]:
        s.wait_event(start)
    sc.st_conv_run_plans_on_streams_many(plans, use, steps)      # the library's issue loop, as for the pipelined fused forms
    for s in use[1:]:
        done = torch.cuda.Event()
        done.record(s)
        use[0].wait_event(done)
    stop.record(use[0])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return wall_ms / steps, start.elapsed_time(stop) / steps


def launch_percentiles(run, policy: str, n: int = 300):
    """p10 / median / p90 of single steps, each bracketed by its own pair of HIP events on the launch stream."""
    import torch
    stream = torch.cuda.Stream()
    for _ in range(20):
        run(policy, stream)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for a, b in ev:
        a.record(stream)
        run(policy, stream)
        b.record(stream)
    torch.cuda.synchronize()
    t = sorted(a.elapsed_time(b) * 1e3 for a, b in ev)
    return {"p10_us": t[n // 10], "median_us": t[n // 2], "p90_us": t[(9 * n) // 10]}


def launch_floor_us(n: int = 2000) -> float:
    import torch
    from paper_1901_00041_amd import st_conv as sc
    stream = torch.cuda.Stream()
    for _ in range(100):
        sc.st_launch_empty(stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(n):
        sc.st_launch_empty(stream)
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / n


def cpu_baseline(cfg: int, budget_s: float = 12.0):
    """The oracle as it stands, timed on this host over whole tenants of the workload until the budget
    is spent (at least one tenant)."""
    from oracle import oracle
    from paper_1901_00041_amd import synth
    if cfg == 5:
        steps = synth.resnet50_steps()
        work = [(5, 0, s.index, s.shape, 2.0) for s in steps]
        label = "configs[4], tenant 0, conv layers in step order"
    else:
        work = [(cfg, t, 0, s, 1.0) for t, s in enumerate(synth.config_shapes(cfg))]
        label = f"configs[{cfg - 1}], whole tenants in order"
    done_flops, spent, n_done = 0, 0.0, 0
    reps = 0
    while spent < budget_s and reps < 1000:
        for (c, t, layer, s, gain) in work:
            x = synth.gen_input(c, t, layer, s).astype("float64")
            w = synth.gen_weight(c, t, layer, s, gain).astype("float64")
            t0 = time.perf_counter()
            oracle.conv2d(x, w, s.stride, s.pad)
            spent += time.perf_counter() - t0
            done_flops += s.flops
            n_done += 1
            if spent >= budget_s:
                break
        reps += 1
    return {"value": done_flops / spent / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{label}: {n_done} layer evaluations, {done_flops / 1e9:.2f} GFLOP in {spent:.1f} s (fp64 direct conv, gcc -O2, OpenMP)"}


def paper_sweep(iters: int = 200, warmup: int = 20):
    """The paper's kernel-level experiment (Section 4.1, Figure 7, Table 1) on this GPU: R same-shape tenants,
    own weights and inputs each, R scaled from 2 to 120, for the three problem shapes of Table 1 expressed as
    convolutions, under the three issue policies.  Reports the speed-up of the fused launch over the next best
    policy at R = 10, R = 20 and as a geometric mean over R, in fp32 (the paper's precision) and bf16."""
    import math
    import torch
    from paper_1901_00041_amd import st_conv as sc
    shapes = {"conv_resnet18 (M=256,N=128,K=1152)": (1, 128, 16, 16, 128, 3, 3, 1, 1),
              "matvec_rnn (512,1,512)": (1, 512, 1, 1, 512, 1, 1, 1, 0),
              "square (256,256,256)": (1, 256, 16, 16, 256, 1, 1, 1, 0)}
    rs = [2, 4, 6, 8, 10, 14, 20, 28, 40, 56, 80, 120]
    streams = [torch.cuda.Stream() for _ in range(max(rs))]
    pipes = {name: sc.Pipeline(depth) for name, (depth, _) in PIPELINED.items()}
    out = {}
    for dtype, tdt in (("f32", torch.float32), ("bf16", torch.bfloat16)):
        for name, (N, C, H, W, K, R_, S_, st, pd) in shapes.items():
            P, Q = (H + 2 * pd - R_) // st + 1, (W + 2 * pd - S_) // st + 1
            rows = []
            for r in rs:
                keep, sets = [], []
                for copy in range(max(d for d, _ in PIPELINED.values())):   # one set of tensors per batch in flight
                    descs = []
                    for t in range(r):
                        x = torch.randn((N, H, W, C), device="cuda").to(tdt)
                        w = (torch.randn((K, R_, S_, C), device="cuda") / (C * R_ * S_) ** 0.5).to(tdt)
                        y = torch.empty((N, P, Q, K), dtype=torch.float32, device="cuda")
                        keep.append((x, w, y))
                        descs.append(sc.make_desc(N, C, H, W, K, R_, S_, st, pd, dtype, "f32", x, w, y))
                    sets.append(descs)
                descs = sets[0]
                plan = sc.st_conv_plan(descs, keep=keep)
                pplans = {name: [sc.st_conv_plan(sets[i], sc.plan_opts(target_items=slots), keep=keep) for i in range(depth)]
                          for name, (depth, slots) in PIPELINED.items()}
                solo = [sc.st_conv_plan([d], keep=keep) for d in descs]
                flops = int(sc.st_conv_plan_info(plan).flops)
                turn = {name: 0 for name in PIPELINED}

                def run(policy, stream, plan=plan, pplans=pplans, solo=solo, r=r, turn=turn):
                    if policy == "fused":
                        sc.st_conv_run(plan, stream)
                    elif policy in PIPELINED:
                        i = turn[policy] = (turn[policy] + 1) % len(pplans[policy])
                        pipes[policy].run(pplans[policy][i])
                    elif policy == "time_only_same_tiles":
                        sc.st_conv_run_time_only(plan, stream)
                    elif policy == "space_only_same_tiles":
                        sc.st_conv_run_space_only(plan, [stream] + streams[1:r])
                    elif policy == "time_only":
                        sc.st_conv_run_plans_time_only(solo, stream)
                    else:
                        sc.st_conv_run_plans_space_only(solo, [stream] + streams[1:r])
                t = {pol: time_policy(run, pol, iters, warmup)[0]
                     for pol in ["fused", "time_only", "space_only", "time_only_same_tiles", "space_only_same_tiles"] +
                     list(PIPELINED)}
                for pol in PIPELINED:
                    t[pol] = min(t[pol], time_pipelined_native(pplans[pol], iters, warmup, tries=1))
                t["fused_single_stream"] = t["fused"]
                t["fused"] = min([t["fused"]] + [t[p] for p in PIPELINED])         # the best form of every policy
                t["space_only_free"] = time_free_running(solo, streams, iters, warmup)[0]
                t["time_only"] = min(t["time_only"], t["time_only_same_tiles"])      # the best form of each baseline
                t["space_only"] = min(t["space_only"], t["space_only_same_tiles"], t["space_only_free"])
                best_other = min(t["time_only"], t["space_only"])
                rows.append({"R": r, "fused_us": t["fused"] * 1e3, "fused_single_stream_us": t["fused_single_stream"] * 1e3,
                             "time_only_us": t["time_only"] * 1e3,
                             "space_only_us": t["space_only"] * 1e3, "fused_tflops": flops / (t["fused"] * 1e-3) / 1e12,
                             "vs_time_only": t["time_only"] / t["fused"], "vs_space_only": t["space_only"] / t["fused"],
                             "vs_next_best": best_other / t["fused"],
                             "next_best": "time_only" if t["time_only"] <= t["space_only"] else "space_only"})
            print(f"paper sweep: {dtype} {name} done", file=sys.stderr, flush=True)
            gm = lambda key: math.exp(sum(math.log(x[key]) for x in rows) / len(rows))
            out[f"{dtype} {name}"] = {"rows": rows, "geomean_vs_time_only": gm("vs_time_only"),
                                      "geomean_vs_space_only": gm("vs_space_only"), "geomean_vs_next_best": gm("vs_next_best"),
                                      "R10_vs_next_best": next(x["vs_next_best"] for x in rows if x["R"] == 10),
                                      "R20_vs_next_best": next(x["vs_next_best"] for x in rows if x["R"] == 20)}
    return {"mode": "paper_sweep", "R": rs, "results": out,
            "paper_table1_V100_fp32": {"conv": {"R10": 1.68, "R20": 2.88, "geomean": 3.23, "next_best": "space_only"},
                                       "matvec": {"R10": 1.21, "R20": 2.14, "geomean": 2.48, "next_best": "time_only"},
                                       "square": {"R10": 2.42, "R20": 2.47, "geomean": 4.93, "next_best": "space_only"},
                                       "conv_geomean_vs_time_only": [7.73, 7.71]}}


def arrival_trace(steps: int = 400, p_ready: float = 0.7, capacity: int = 256, seed: int = 11):
    """Dynamic arrival (Section 4: the scheduler merges whichever kernels are ready and caches the merged
    kernels): a pool of 8 tenants (configs[1]'s four layers and four of configs[2]'s), a seeded Bernoulli ready
    set per step, plans from the plan cache.  Reports the host time of the cache call (hit / miss), the hit rate,
    and the whole trace's throughput against launching every ready tenant on its own (time-only, per-tenant
    plans)."""
    import numpy as np
    import torch
    from paper_1901_00041_amd import st_conv as sc
    from paper_1901_00041_amd import synth
    dt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
    shapes = synth.config_shapes(2) + synth.config_shapes(3)[:4]
    keep, descs = [], []
    for t, s in enumerate(shapes):
        x = torch.randn((s.N, s.H, s.W, s.C), device="cuda").to(dt[s.dtype])
        w = (torch.randn((s.K, s.R, s.S, s.C), device="cuda") / (s.C * s.R * s.S) ** 0.5).to(dt[s.dtype])
        y = torch.empty((s.N, s.P, s.Q, s.K), dtype=dt[s.out_dtype], device="cuda")
        keep.append((x, w, y))
        descs.append(sc.make_desc(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, s.dtype, s.out_dtype, x, w, y))
    rng = np.random.default_rng(seed)
    trace = []
    for _ in range(steps):
        ready = [t for t in range(len(shapes)) if rng.random() < p_ready] or [int(rng.integers(len(shapes)))]
        trace.append(ready)
    flops = sum(shapes[t].flops for ready in trace for t in ready)
    stream = torch.cuda.Stream()
    out = {"mode": "arrival_trace", "pool_tenants": len(shapes), "steps": steps, "p_ready": p_ready,
           "cache_capacity": capacity, "distinct_ready_sets": len({tuple(r) for r in trace}),
           "mean_ready": sum(len(r) for r in trace) / steps, "flops": flops}
    # fused, through the cache: first pass cold (misses build plans), second pass warm
    cache = sc.PlanCache(capacity)
    for label in ("cold", "warm"):
        t_hit, t_miss = [], []
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for ready in trace:
            h0 = time.perf_counter()
            plan, hit = cache.get([descs[t] for t in ready], stream)
            (t_hit if hit else t_miss).append((time.perf_counter() - h0) * 1e6)
            sc.st_conv_run(plan, stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        out[f"fused_{label}"] = {"us_per_step": wall / steps * 1e6, "tflops": flops / wall / 1e12,
                                 "hits": len(t_hit), "misses": len(t_miss),
                                 "host_us_hit_median": statistics.median(t_hit) if t_hit else None,
                                 "host_us_miss_median": statistics.median(t_miss) if t_miss else None}
    st = cache.stats()
    out["cache"] = {"hits": int(st.hits), "misses": int(st.misses), "evictions": int(st.evictions), "size": int(st.size)}
    # the same trace with four steps in flight: a ring of four streams, each with its own tensors and its own plan cache
    # (a plan must not run twice at once), plans made for a quarter of the GPU
    depth = 4
    pipe = sc.Pipeline(depth)
    rings = []
    for _ in range(depth):
        rk, rd = [], []
        for (x, w, y), s in zip(keep[:len(shapes)], shapes):
            x2, w2, y2 = x.clone(), w.clone(), torch.empty_like(y)
            rk.append((x2, w2, y2))
            rd.append(sc.make_desc(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, s.dtype, s.out_dtype, x2, w2, y2))
        rings.append((sc.PlanCache(capacity, sc.plan_opts(target_items=pipe.slots)), rd, rk))
    for label in ("cold", "warm"):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i, ready in enumerate(trace):
            cache_i, rd, _ = rings[i % depth]
            stream = pipe.next()
            plan, _hit = cache_i.get([rd[t] for t in ready], stream)
            sc.st_conv_run(plan, stream)
        pipe.sync()
        wall = time.perf_counter() - t0
        out[f"fused_pipelined4_{label}"] = {"us_per_step": wall / steps * 1e6, "tflops": flops / wall / 1e12}
    for c, _, _ in rings:
        c.destroy()
    # baseline: every ready tenant on its own, per-tenant plans built once
    solo = [sc.st_conv_plan([d], keep=keep) for d in descs]
    for _ in range(2):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for ready in trace:
            sc.st_conv_run_plans_time_only([solo[t] for t in ready], stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    out["time_only"] = {"us_per_step": wall / steps * 1e6, "tflops": flops / wall / 1e12}
    out["speedup_vs_time_only_warm"] = out["time_only"]["us_per_step"] / out["fused_warm"]["us_per_step"]
    out["speedup_pipelined4_vs_time_only_warm"] = out["time_only"]["us_per_step"] / out["fused_pipelined4_warm"]["us_per_step"]
    cache.destroy()
    return out


def isolation(reps: int = 30):
    """Predictability (Section 3 observes that identical models sharing a GPU under spatial multiplexing finish up
    to 25% apart): R identical tenants (the Section 4.1 convolution, own weights and inputs each); per-tenant
    completion time inside one fused launch (in-kernel clock, per work-list order) and under the space-only
    policy (one stream per tenant, HIP events).  gap = (slowest - fastest) / slowest over the tenants' mean
    completion times."""
    import numpy as np
    import torch
    from paper_1901_00041_amd import st_conv as sc
    out = {"mode": "isolation", "shape": "3x3 128->128 @16x16 (M=256, N=128, K=1152), bf16 in / fp32 out", "results": {}}
    for R in (8, 32):
        keep, descs = [], []
        for t in range(R):
            x = torch.randn((1, 16, 16, 128), device="cuda").to(torch.bfloat16)
            w = (torch.randn((128, 3, 3, 128), device="cuda") / 1152 ** 0.5).to(torch.bfloat16)
            y = torch.empty((1, 16, 16, 128), dtype=torch.float32, device="cuda")
            keep.append((x, w, y))
            descs.append(sc.make_desc(1, 128, 16, 16, 128, 3, 3, 1, 1, "bf16", "f32", x, w, y))
        res = {}
        for label, order in (("fused_longest_first", 0), ("fused_equal_progress", 2)):
            plan = sc.st_conv_plan(descs, sc.plan_opts(order=order), keep=keep)
            for _ in range(3):
                sc.st_conv_run(plan)
            torch.cuda.synchronize()
            ends = np.stack([sc.st_conv_run_tenant_times(plan)[1] for _ in range(reps)]).astype(np.float64) / 1e3
            mean = ends.mean(axis=0)
            res[label] = {"completion_us_fastest": float(mean.min()), "completion_us_slowest": float(mean.max()),
                          "gap": float((mean.max() - mean.min()) / mean.max()),
                          "work_items": int(sc.st_conv_plan_info(plan).n_items)}
        solo = [sc.st_conv_plan([d], keep=keep) for d in descs]
        streams = [torch.cuda.Stream() for _ in range(R)]
        ends = np.zeros((reps, R))
        for rep in range(reps + 3):
            start = torch.cuda.Event(enable_timing=True)
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(R)]
            start.record(streams[0])
            for t in range(R):
                streams[t].wait_event(start)
                sc.st_conv_run(solo[t], streams[t])
                evs[t].record(streams[t])
            torch.cuda.synchronize()
            if rep >= 3:
                ends[rep - 3] = [start.elapsed_time(e) * 1e3 for e in evs]
        mean = ends.mean(axis=0)
        res["space_only"] = {"completion_us_fastest": float(mean.min()), "completion_us_slowest": float(mean.max()),
                             "gap": float((mean.max() - mean.min()) / mean.max())}
        out["results"][f"R={R}"] = res
    out["paper_context"] = "MPS on a V100: identical ResNet-50 models finish up to 25% apart (Section 3)"
    return out


def probes():
    """Sustained rates of one compute unit's data paths (st_probe_cu_path): what a K step that stages its operands
    through LDS can at best move per clock."""
    from paper_1901_00041_amd import st_conv as sc
    names = {0: "LDS write (ds_write_b128)", 1: "LDS read (ds_read_b128)", 2: "global -> VGPR -> LDS write, barrier per round",
             3: "global -> LDS direct (global_load_lds_dwordx4)"}
    out = {"mode": "probes", "unit": "bytes per shader clock per compute unit", "results": {}}
    for m, name in names.items():
        out["results"][name] = {"one_workgroup": sc.st_probe_cu_path(m, 1), "two_workgroups": sc.st_probe_cu_path(m, 2)}
    out["chip"] = achievable_roofs()
    return out


def achievable_roofs():
    """What this chip reaches on a plain copy and on a register-only MFMA loop (st_probe_chip), beside the published
    peaks the roofline is priced against."""
    from paper_1901_00041_amd import st_conv as sc
    return {"hbm_copy_GBps": sc.st_probe_chip(0) / 1e9, "mfma_bf16_TFLOPs": sc.st_probe_chip(1) / 1e12,
            "mfma_f16_TFLOPs": sc.st_probe_chip(2) / 1e12, "mfma_f32_TFLOPs": sc.st_probe_chip(3) / 1e12,
            "published": {"hbm_GBps": PEAK_HBM_GBS, "mfma_bf16_TFLOPs": PEAK_BF16_TFLOPS, "mfma_f32_TFLOPs": PEAK_F32_TFLOPS}}


def measured_traffic(cfg: int):
    """HBM bytes per fused launch from the committed counter summary (profiles/hbm_traffic.txt), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 3 and f[0] == str(cfg):
                return float(f[1]) + float(f[2])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--no-sweep", action="store_true", help="skip the other configurations")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the cold-cache variant and the per-launch percentiles (keeps a kernel trace of the run "
                         "to the launches of the three policies)")
    ap.add_argument("--paper-sweep", action="store_true",
                    help="run the paper's R-sweep of its three Table-1 shapes instead of the headline benchmark")
    ap.add_argument("--arrival-trace", action="store_true",
                    help="run a synthetic trace whose ready set of tenants changes every step, through the plan cache")
    ap.add_argument("--isolation", action="store_true",
                    help="per-tenant completion spread of identical tenants: fused launch vs space-only")
    ap.add_argument("--probes", action="store_true", help="measure the compute unit's LDS and vector-memory path rates")
    ap.add_argument("--counters", action="store_true",
                    help="counter-collection mode for rocprofv3 --pmc: only K fused steps of the workload and K launches of "
                         "a 64 MiB copy kernel (the known-traffic reference); prints a short JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (tenants are independent; sharding is placement only). "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1901_00041_amd import st_conv as sc
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    sc.lib()
    torch.cuda.set_device(0)
    steps = args.steps if args.steps is not None else (200 if args.config == 5 else 2000)
    warmup = args.warmup if args.warmup is not None else (20 if args.config == 5 else 200)

    if args.paper_sweep:
        print(json.dumps(paper_sweep()))
        return
    if args.arrival_trace:
        print(json.dumps(arrival_trace()))
        return
    if args.isolation:
        print(json.dumps(isolation()))
        return
    if args.probes:
        print(json.dumps(probes()))
        return
    if args.counters:
        run, flops, nbytes, n_launch, meta = build_workload(args.config)
        k = args.steps if args.steps is not None else 20
        src = torch.empty(64 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(k):
            run("fused", None)
        for _ in range(k):
            sc.st_launch_copy(src, dst, src.numel(), None)
        torch.cuda.synchronize()
        print(json.dumps({"mode": "counters", "workload": CONFIG_TEXT[args.config], "fused_steps": k,
                          "conv_launches_per_step": n_launch, "algorithmic_bytes_per_step": nbytes, "flops_per_step": flops,
                          "copy_launches": k, "copy_bytes_read": src.numel(), "copy_bytes_written": src.numel()}))
        return

    floor_us = launch_floor_us()

    def measure(cfg: int, k: int, w: int):
        # enough copies of the tensors to exceed the 256 MB memory-side cache several times over
        copies = 1 if cfg == 5 else max(4, int(1.2e9 // max(1, {1: 475e3, 2: 8.52e6, 3: 14.25e6, 4: 104.4e6}[cfg])))
        copies = 1 if args.no_extras else min(copies, 160)
        run, flops, nbytes, n_launch, meta = build_workload(cfg, copies)
        out = {"flops": flops, "algorithmic_bytes": nbytes, "plan_build_us": round(meta["plan_build_us"], 1),
               "work_items": meta["n_items"], "fused_launches_per_step": n_launch}
        pols = ["fused", "time_only", "space_only"] + (["time_only_retuned", "space_only_retuned"] if meta.get("retuned") else [])
        if meta.get("chains"):
            pols.append("space_only_chains")     # every tenant's whole chain on its own stream, joined once at the end
            pols.append("fused_groups2")         # two tenant groups, each a chain of fused launches on its own stream
        if not args.no_extras:
            pols += list(meta.get("pipelined", []))   # the fused launch with several independent batches in flight
        for pol in pols:
            wall_ms, ev_ms = time_policy(run, pol, k, w)
            if pol in ("space_only_chains", "fused_groups2"):
                # which hardware queue a stream lands on varies from run to run (four queues for nine streams); give
                # this baseline the best of three tries
                for _ in range(2):
                    wall_ms, ev_ms = min((wall_ms, ev_ms), time_policy(run, pol, k, w))
            if pol in PIPELINED:
                # the same for the pipelined forms: two more tries on freshly created streams
                for _ in range(2):
                    meta["new_streams"](pol)
                    wall_ms, ev_ms = min((wall_ms, ev_ms), time_policy(run, pol, k, w))
                if cfg != 5:
                    wall_ms = min(wall_ms, time_pipelined_native(meta["keep"][5][pol], k, w))
            out[pol] = {"ms_per_step": wall_ms, "event_ms_per_step": None if pol in PIPELINED else ev_ms,
                        "tflops": flops / (wall_ms * 1e-3) / 1e12}
        if cfg != 5:
            # free-running streams: per-tenant plans, no joins between steps (the strongest form of space-only)
            plan, keep, streams, solo, cold_plans = meta["keep"][:5]
            wall_ms, ev_ms = min(time_free_running(solo, streams, k, w),
                                 time_free_running(solo, [torch.cuda.Stream() for _ in streams], k, w),
                                 time_free_running(solo, [torch.cuda.Stream() for _ in streams], k, w))   # three sets of streams
            out["space_only_free"] = {"ms_per_step": wall_ms, "event_ms_per_step": ev_ms, "tflops": flops / (wall_ms * 1e-3) / 1e12}
            pols = pols + ["space_only_free"]
        # headline speed-ups are against the best form of each baseline (same tiles as the fused plan, each tenant
        # planned alone, streams joined per step or free-running)
        t_time = min(out[p]["ms_per_step"] for p in pols if p.startswith("time_only"))
        t_space = min(out[p]["ms_per_step"] for p in pols if p.startswith("space_only"))
        forms = [p for p in pols if p.startswith("fused") or p in PIPELINED]
        t_fused = min(out[p]["ms_per_step"] for p in forms)
        out["best"] = {"ms_per_step": t_fused, "tflops": flops / (t_fused * 1e-3) / 1e12,
                       "form": min(forms, key=lambda p: out[p]["ms_per_step"])}
        out["speedup_vs_time_only"] = t_time / t_fused
        out["speedup_vs_space_only"] = t_space / t_fused
        # one batch at a time: a single fused launch sequence against per-tenant launches that are joined every step
        t_single = min(out[p]["ms_per_step"] for p in ("fused", "fused_groups2") if p in out)
        out["speedup_single_batch"] = {
            "vs_time_only": t_time / t_single,
            "vs_space_only": min(out[p]["ms_per_step"] for p in pols if p.startswith("space_only") and p not in
                                 ("space_only_free", "space_only_chains")) / t_single}
        out["pct_bf16_mfma_peak"] = 100.0 * out["best"]["tflops"] / PEAK_BF16_TFLOPS
        if not args.no_extras:
            out["fused"].update(launch_percentiles(run, "fused", 100 if cfg == 5 else 300))
        if cfg == 5:
            # glue inside the pass: the one max-pool launch over all tenants' stem outputs (the residual adds and
            # ReLUs are in the conv epilogues).  Timed alone, back to back on one stream.
            stack = meta["keep"]
            st0 = stack.steps[0]
            s0 = st0.shape

            def pool_only(policy, stream):
                sc.st_maxpool_nhwc(stack.buf[st0.dst], stack.buf[st0.pool_dst], stack.n_tenants * s0.N, s0.P, s0.Q, s0.K, 3, 2, 1,
                                   "bf16", stream)
            pool_ms = time_policy(pool_only, "pool", 200, 20)[1]
            out["glue"] = {"maxpool_ms_per_pass": pool_ms, "conv_only_ms_per_pass": out["fused"]["event_ms_per_step"] - pool_ms,
                           "end_to_end_ms_per_pass": out["fused"]["event_ms_per_step"],
                           "note": "back-to-back pooling launches; inside the pass the launch also pays the stream's serialisation"}
        if cfg == 5 and not args.no_extras:
            # tenants at different depths of the network (offsets spread evenly): every launch mixes eight different
            # layers; the baselines issue the same launches' work per tenant-layer.  One cycle = the work of one pass.
            stag = {}
            for pol in ("fused", "time_only", "space_only"):
                wall_ms, ev_ms = time_policy(run, pol + "_staggered", max(3, k // 2), 2)
                stag[pol] = {"ms_per_step": wall_ms, "tflops": flops / (wall_ms * 1e-3) / 1e12}
            stag["speedup_vs_time_only"] = stag["time_only"]["ms_per_step"] / stag["fused"]["ms_per_step"]
            stag["speedup_vs_space_only"] = stag["space_only"]["ms_per_step"] / stag["fused"]["ms_per_step"]
            stag["offsets"] = list(meta["keep"].stagger_offsets)
            stag["work_items"] = int(meta["keep"].n_items_staggered)
            out["staggered"] = stag
        if meta.get("copies", 1) > 1:
            wall_ms, ev_ms = time_policy(run, "fused_cold", k, w)
            out["fused_cold"] = {"ms_per_step": wall_ms, "event_ms_per_step": ev_ms, "tflops": flops / (wall_ms * 1e-3) / 1e12,
                                 "tensor_copies": meta["copies"], "rotated_bytes": meta["copies"] * nbytes}
        return out

    head = measure(args.config, steps, warmup)
    fused = head["fused"]
    # roofline of the dominant kernel (the fused conv kernel), from HIP events on its stream
    ev_s = fused["event_ms_per_step"] * 1e-3 / head["fused_launches_per_step"]
    ai = head["flops"] / head["algorithmic_bytes"]
    ridge = PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    if args.config == 1:
        ridge = PEAK_F32_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    if ai >= ridge:
        peak = PEAK_F32_TFLOPS if args.config == 1 else PEAK_BF16_TFLOPS
        ach = head["flops"] / head["fused_launches_per_step"] / ev_s / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak, "traffic": None}
    else:
        ach = head["algorithmic_bytes"] / head["fused_launches_per_step"] / ev_s / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                "traffic": None}
    roof["traffic"] = measured_traffic(args.config)
    roof["kernel"] = "st_conv_kernel (fused launch)"
    roof["avg_launch_us"] = ev_s * 1e6
    roof["arithmetic_intensity"] = ai
    # the same ratio at the job's throughput (several launches in flight overlap; a launch's own duration does not
    # shrink): algorithmic bytes or flops per step / time per step of the best form
    per_s = (head["flops"] / 1e12 if roof["bound"] == "mfma" else head["algorithmic_bytes"] / 1e9) / (head["best"]["ms_per_step"] * 1e-3)
    if not args.no_extras:
        roof["achievable"] = achievable_roofs()
    roof["achieved_at_throughput"] = per_s
    roof["frac_at_throughput"] = per_s / roof["peak"]

    per_config = {}
    if not args.no_sweep:
        for cfg in (1, 2, 3, 4, 5):
            if cfg == args.config:
                per_config[str(cfg)] = head
                continue
            try:
                per_config[str(cfg)] = measure(cfg, 40 if cfg == 5 else 500, 5 if cfg == 5 else 50)
            except Exception as e:  # a configuration that cannot run is reported, not hidden
                per_config[str(cfg)] = {"error": repr(e)}
        ok = [v for v in per_config.values() if "error" not in v]
        if ok:
            import math
            per_config["geomean_speedup_vs_time_only"] = math.exp(sum(math.log(v["speedup_vs_time_only"]) for v in ok) / len(ok))
            per_config["geomean_speedup_vs_space_only"] = math.exp(sum(math.log(v["speedup_vs_space_only"]) for v in ok) / len(ok))

    line = {
        "metric": "aggregate conv TFLOP/s (% bf16 MFMA peak) + speedup vs time-only/space-only",
        "value": head["best"]["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": head["best"]["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if args.config == 1 else "bf16", "data": "synthetic",
        "config": {"workload": CONFIG_TEXT[args.config], "policy": policy_text(head["best"]["form"]),
                   "tenants": __import__("paper_1901_00041_amd.synth", fromlist=["x"]).N_TENANTS[args.config]},
        "pct_bf16_mfma_peak": head["pct_bf16_mfma_peak"],
        "speedup_vs_time_only": head["speedup_vs_time_only"], "speedup_vs_space_only": head["speedup_vs_space_only"],
        "speedup_single_batch": head["speedup_single_batch"],
        "policies": {k: head[k] for k in ("fused", "fused_cold", "time_only", "space_only", "time_only_retuned",
                                          "space_only_retuned", "space_only_chains", "space_only_free", "fused_groups2",
                                          "fused_pipelined", "fused_pipelined4") if k in head},
        "launch_floor_us": floor_us, "plan_build_us": head["plan_build_us"], "work_items": head["work_items"],
        "gpu_max_hw_queues": os.environ.get("GPU_MAX_HW_QUEUES", "default(4)"),
        "roofline": roof,
        "paper_context": PAPER_CONTEXT,
    }
    for extra in ("staggered", "glue"):
        if extra in head:
            line[extra] = head[extra]
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(args.config)
    if per_config:
        line["per_config"] = {k: (v if not isinstance(v, dict) else {kk: vv for kk, vv in v.items() if kk != "keep"})
                              for k, v in per_config.items()}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
