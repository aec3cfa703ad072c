#!/usr/bin/env python3
"""Benchmark of the fused multi-tenant convolution path on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--no-sweep] [--no-cpu] [--no-extras]
                  [--policies fused,time_only,...]

One PASS is the whole hot path over one batch of synthetic input: every tenant's layer (configurations 1-4), or
every tenant's 53-layer stack (configuration 5), through cached plans, tensors resident in HBM.  One STEP is
`passes_per_step` passes issued back to back on one stream (reported in `config`), sized so that a step takes
10-20 ms and a handful of steps is a stable measurement.  Exactly K steps are timed between two device
synchronisations; every step is also bracketed by HIP events on the launch stream (median, p10, p90).

Prints ONE JSON line.  `value` is the aggregate conv TFLOP/s of the fused (space-time) policy on the headline
workload, one batch at a time on one stream, in the form named by `config.policy` (a fixed choice, not a minimum
over forms).  The time-only and space-only baselines are timed the same way (one batch at a time, per-tenant
launches joined at every layer), once with the fused plan's tiles and once with each tenant planned alone; the
speed-ups are against the FASTER of the two.  Forms with several batches in flight, free-running streams and
cold caches are under `extras` and never enter `value`.  `roofline` describes the launches `value` timed;
`per_config` carries the same measurement for every configuration with its own roofline bound; `cpu_baseline`
is the fp64 oracle timed on this host.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import statistics
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6     # MI355X dense bf16/fp16 MFMA
PEAK_F32_TFLOPS = 157.3       # MI355X fp32 matrix
PEAK_HBM_GBS = 8000.0
HEADLINE_CONFIG = 5           # configs[4]: the largest single-GPU configuration
# passes per step: a step lasts 10-20 ms for the fused policy
PASSES_PER_STEP = {1: 2048, 2: 2048, 3: 1024, 4: 256, 5: 40}
# the form of the fused policy that `value` reports, per configuration (fixed; every other form is an extra):
# one fused launch per pass for the single-layer configurations, and for the 53-layer stacks one persistent launch
# per pass (the layer-by-layer form, 49 fused launches per pass, is timed beside it as "fused")
HEADLINE_FORM = {1: "fused", 2: "fused", 3: "fused", 4: "fused", 5: "fused_chain"}
BASELINES = ["time_only", "space_only", "time_only_retuned", "space_only_retuned"]
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
POLICY_TEXT = {
    "fused": "fused space-time launches on one stream, cached plans, one batch at a time",
    "fused_chain": "fused space-time policy as ONE persistent launch per pass: every tenant's layers in work queues (per XCD), "
                   "a layer's tiles start when that tenant's previous layer is complete; one stream, one batch at a time",
}


# ----------------------------------------------------------------------------------------------------------------
# workloads
# ----------------------------------------------------------------------------------------------------------------
class Workload:
    """run(form, stream) issues ONE pass of the given form; forms lists what exists."""

    def __init__(self, cfg: int, copies: int = 1):
        import torch
        from paper_1901_00041_amd import st_conv as sc
        from paper_1901_00041_amd import synth
        self.cfg, self.sc, self.torch = cfg, sc, torch
        self.copies = copies
        if cfg == 5:
            from paper_1901_00041_amd.stack import ResNetStack
            self.stack = ResNetStack(n_tenants=synth.N_TENANTS[5], cfg=5)
            self.flops, self.bytes = self.stack.flops, self.stack.bytes
            self.plan_build_us = self.stack.plan_build_us
            self.launches = {"fused": self.stack.n_launches, "fused_chain": 1}
            self.n_items = self.stack.n_items
            # per fused launch: (flops, algorithmic bytes), for the configuration's own roofline bound
            self.launch_work = [(int(sc.st_conv_plan_info(p).flops), int(sc.st_conv_plan_info(p).bytes)) for p in self.stack.group_plans]
            self.forms = ["fused", "time_only", "space_only", "time_only_retuned", "space_only_retuned"]
            self.forms.insert(0, "fused_chain")       # the whole pass as one persistent launch
            self.extra_forms = ["fused_chain2", "fused_groups2", "space_only_chains", "fused_staggered", "time_only_staggered", "space_only_staggered"] + list(PIPELINED)
            self.passes_per_run = {"fused_chain2": 2}      # one persistent launch over two independent batches
            self._twins, self._pipes, self._turn = {}, {}, {}
            return
        dt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
        shapes = synth.config_shapes(cfg)
        self.shapes = shapes
        keep, sets = [], []
        for c in range(copies):
            descs = []
            for t, s in enumerate(shapes):
                if c == 0:
                    x = torch.from_numpy(synth.gen_input(cfg, t, 0, s).transpose(0, 2, 3, 1).copy()).to(dt[s.dtype]).cuda()
                    w = torch.from_numpy(synth.gen_weight(cfg, t, 0, s).transpose(0, 2, 3, 1).copy()).to(dt[s.dtype]).cuda()
                else:
                    x, w = keep[t][0].clone(), keep[t][1].clone()
                y = torch.empty((s.N, s.P, s.Q, s.K), dtype=dt[s.out_dtype], device="cuda")
                keep.append((x, w, y))
                descs.append(sc.make_desc(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, s.dtype, s.out_dtype, x, w, y))
            sets.append(descs)
        self.keep, self.sets = keep, sets
        t_plan = []
        for _ in range(5):
            t0 = time.perf_counter()
            self.plan = sc.st_conv_plan(sets[0], keep=keep)
            t_plan.append((time.perf_counter() - t0) * 1e6)
        self.plan_build_us = statistics.median(t_plan)
        info = sc.st_conv_plan_info(self.plan)
        self.flops, self.bytes, self.n_items = int(info.flops), int(info.bytes), int(info.n_items)
        self.launches = {"fused": 1}
        self.launch_work = [(self.flops, self.bytes)]
        self.streams = [torch.cuda.Stream() for _ in shapes]
        self.solo = [sc.st_conv_plan([d], keep=keep) for d in sets[0]]      # each tenant planned alone (retuned baselines)
        self.forms = ["fused", "time_only", "space_only", "time_only_retuned", "space_only_retuned"]
        self.extra_forms = ["space_only_free"]
        self.cold_plans, self.pipe_plans, self._turn = [], {}, {"cold": 0}
        if copies > 1:
            self.cold_plans = [self.plan] + [sc.st_conv_plan(d, keep=keep) for d in sets[1:]]
            self.extra_forms.append("fused_cold")
            for name, (depth, slots) in PIPELINED.items():
                if copies >= depth:
                    self.pipe_plans[name] = [sc.st_conv_plan(sets[i], sc.plan_opts(target_items=slots), keep=keep) for i in range(depth)]
                    self.extra_forms.append(name)

    def run(self, form: str, stream) -> None:
        sc = self.sc
        if self.cfg == 5:
            if form == "fused_chain2":
                # two independent batches (16 sequences, two per XCD) in ONE persistent launch: while one tenant's
                # stage boundary is in flight, the XCD's other tenant has tiles to run
                if form not in self._twins:
                    from paper_1901_00041_amd.stack import ResNetStack
                    twins = [ResNetStack(n_tenants=self.stack.n_tenants, cfg=5, seeded_weights=False) for _ in range(2)]
                    ops = []
                    for b, tw in enumerate(twins):
                        tw.build_chain()
                        ops += [sc.make_chain_op(o.kind, o.sequence + b * tw.n_tenants, o.stage, o.conv) for o in tw.chain_ops]
                    self._twins[form] = (twins, sc.Chain(ops, None, keep=twins))
                self._twins[form][1].run(stream)
                return
            if form in PIPELINED:
                from paper_1901_00041_amd.stack import ResNetStack
                depth, slots = PIPELINED[form]
                if form not in self._twins:
                    self._twins[form] = [ResNetStack(n_tenants=self.stack.n_tenants, cfg=5, seeded_weights=False,
                                                     plan_opts=sc.plan_opts(target_items=slots)) for _ in range(depth)]
                    self._pipes[form] = sc.Pipeline(depth)
                    self._turn[form] = 0
                i = self._turn[form] = (self._turn[form] + 1) % depth
                self._twins[form][i].run("fused", self._pipes[form].next())
                return
            self.stack.run(form, stream)
            return
        if form == "fused":
            sc.st_conv_run(self.plan, stream)
        elif form == "fused_cold":
            i = self._turn["cold"] = (self._turn["cold"] + 1) % len(self.cold_plans)
            sc.st_conv_run(self.cold_plans[i], stream)
        elif form == "time_only":
            sc.st_conv_run_time_only(self.plan, stream)
        elif form == "space_only":
            sc.st_conv_run_space_only(self.plan, [stream] + self.streams[1:])
        elif form == "time_only_retuned":
            sc.st_conv_run_plans_time_only(self.solo, stream)
        elif form == "space_only_retuned":
            sc.st_conv_run_plans_space_only(self.solo, [stream] + self.streams[1:])
        else:
            raise ValueError(form)

    def check(self, form: str) -> None:
        """After a timed region: a persistent launch that gave up on a dependency wait makes the run fail."""
        chain = None
        if self.cfg == 5 and form == "fused_chain":
            chain = getattr(self.stack, "chain", None)
        elif self.cfg == 5 and form == "fused_chain2" and form in self._twins:
            chain = self._twins[form][1]
        if chain is not None and chain.aborted():
            raise RuntimeError("the chain launch abandoned a pass (dependency wait expired); its timing is void")

    def sync_extra(self, form: str) -> None:
        if self.cfg == 5 and form in self._pipes:
            self._pipes[form].sync()


def time_form(wl: Workload, form: str, steps: int, warmup: int, passes: int):
    """Exactly `steps` steps of `passes` passes each on one stream: wall clock between two device synchronisations,
    plus one HIP event per step boundary on the launch stream."""
    torch = wl.torch
    stream = torch.cuda.Stream()
    for _ in range(warmup * passes):
        wl.run(form, stream)
    wl.sync_extra(form)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    ev[0].record(stream)
    for k in range(steps):
        for _ in range(passes):
            wl.run(form, stream)
        ev[k + 1].record(stream)
    wl.sync_extra(form)
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t0
    wl.check(form)
    per_step_ms = sorted(ev[k].elapsed_time(ev[k + 1]) for k in range(steps))
    pick = lambda q: per_step_ms[min(steps - 1, int(q * steps))]
    ms_per_step = wall_s * 1e3 / steps
    return {"ms_per_step": ms_per_step, "us_per_pass": ms_per_step * 1e3 / passes,
            "event_ms_per_step": {"median": statistics.median(per_step_ms), "p10": pick(0.1), "p90": pick(0.9)},
            "event_us_per_pass_median": statistics.median(per_step_ms) * 1e3 / passes,
            "timed_region_s": wall_s, "tflops": wl.flops * passes * steps / wall_s / 1e12}


def time_pipelined_native(wl: Workload, form: str, steps: int, warmup: int, passes: int):
    """Configurations 1-4, several batches in flight: the library's own issue loop (st_pipeline_run_many) over
    `depth` streams."""
    sc = wl.sc
    plans = wl.pipe_plans[form]
    depth = len(plans)
    pipe = sc.Pipeline(depth)
    pipe.run_many(plans, max(1, warmup * passes // depth))
    pipe.sync()
    t0 = time.perf_counter()
    pipe.run_many(plans, steps * passes // depth)
    pipe.sync()
    wall_s = time.perf_counter() - t0
    n = (steps * passes // depth) * depth
    pipe.destroy()
    return {"us_per_pass": wall_s * 1e6 / n, "tflops": wl.flops * n / wall_s / 1e12, "timed_region_s": wall_s}


def time_free_running(wl: Workload, steps: int, warmup: int, passes: int):
    """Space-only without per-layer joins (configurations 1-4): tenant t's launches back to back on stream t, one fork
    before the first launch and one join after the last."""
    torch, sc = wl.torch, wl.sc
    use = wl.streams
    sc.st_conv_run_plans_on_streams_many(wl.solo, use, warmup * passes)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start = torch.cuda.Event()
    start.record(use[0])
    for s in use[1:]:
        s.wait_event(start)
    sc.st_conv_run_plans_on_streams_many(wl.solo, use, steps * passes)
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t0
    n = steps * passes
    return {"us_per_pass": wall_s * 1e6 / n, "tflops": wl.flops * n / wall_s / 1e12, "timed_region_s": wall_s}


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


# ----------------------------------------------------------------------------------------------------------------
# roofline
# ----------------------------------------------------------------------------------------------------------------
def measured_traffic(cfg: int, form: str):
    """HBM bytes per launch of the dominant kernel from the committed counter summary (profiles/hbm_traffic.txt:
    config, form, bytes read, bytes written), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 4 and f[0] == str(cfg) and f[1] == form:
                return float(f[2]) + float(f[3])
    except OSError:
        pass
    return None


def roofline(wl: Workload, form: str, timing: dict) -> dict:
    """Roofline of the dominant kernel for the launches that `timing` covers.  achieved = algorithmic bytes (or
    FLOPs) of one launch / average launch duration, where the average launch duration is the HIP-event time of the
    timed region on the launch stream divided by the number of launches of that kernel in it.  `bound_us` is the
    configuration's own bound per pass: sum over the pass's fused launches of max(FLOPs / MFMA peak, bytes / HBM
    peak), and `frac_of_own_bound` = bound_us / measured us per pass."""
    cfg = wl.cfg
    peak_tf = PEAK_F32_TFLOPS if cfg == 1 else PEAK_BF16_TFLOPS
    n_launch = wl.launches.get(form, wl.launches["fused"])
    pass_s = timing["event_us_per_pass_median"] * 1e-6
    launch_s = pass_s / n_launch
    t_mfma = wl.flops / (peak_tf * 1e12)
    t_hbm = wl.bytes / (PEAK_HBM_GBS * 1e9)
    bound_us = sum(max(f / (peak_tf * 1e12), b / (PEAK_HBM_GBS * 1e9)) for f, b in wl.launch_work) * 1e6
    if t_mfma >= t_hbm:
        ach = wl.flops / n_launch / launch_s / 1e12
        out = {"bound": "mfma", "achieved": ach, "peak": peak_tf, "unit": "TFLOP/s", "frac": ach / peak_tf}
    else:
        ach = wl.bytes / n_launch / launch_s / 1e9
        out = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS}
    out.update({"traffic": measured_traffic(cfg, form), "kernel": "st_chain_kernel" if form == "fused_chain" else "st_conv_kernel",
                "form": form, "launches_per_pass": n_launch, "avg_launch_us": launch_s * 1e6,
                "algorithmic_bytes_per_launch": wl.bytes / n_launch, "flops_per_launch": wl.flops / n_launch,
                "arithmetic_intensity": wl.flops / wl.bytes, "bound_us_per_pass": bound_us,
                "frac_of_own_bound": bound_us / (pass_s * 1e6),
                "pct_bf16_mfma_peak": 100.0 * wl.flops / pass_s / 1e12 / PEAK_BF16_TFLOPS})
    return out


# ----------------------------------------------------------------------------------------------------------------
# the oracle on this host
# ----------------------------------------------------------------------------------------------------------------
def _oracle_chain(tenant: int, budget_s: float):
    """Tenant `tenant`'s whole 53-layer stack through the oracle, with activations rounded to bf16 wherever the data
    path stores them (after every layer's ReLU, the projection output included).  Returns (final activation NCHW
    float64, seconds spent inside oracle.conv2d, FLOPs done, layers done); stops early once budget_s is spent."""
    import numpy as np
    from oracle import oracle
    from paper_1901_00041_amd import synth
    steps = synth.resnet50_steps()
    buf = {0: synth.gen_input(5, tenant, 0, steps[0].shape).astype(np.float64)}
    spent, flops, done = 0.0, 0, 0
    for st in steps:
        s = st.shape
        w = synth.gen_weight(5, tenant, st.index, s, 2.0).astype(np.float64)
        t0 = time.perf_counter()
        y = oracle.conv2d(buf[st.src], w, s.stride, s.pad)
        spent += time.perf_counter() - t0
        flops += s.flops
        done += 1
        if st.res is not None:
            y = y + buf[st.res]
        if st.relu:
            y = oracle.relu(y)
        buf[st.dst] = oracle.round_bf16(y)
        if st.pool_after:
            buf[st.pool_dst] = oracle.maxpool2d(buf[st.dst], 3, 2, 1)
        if spent >= budget_s:
            break
    last = steps[-1]
    return (buf.get(last.dst) if done == len(steps) else None), spent, flops, done


def cpu_baseline(cfg: int, wl: Workload | None, budget_s: float = 12.0):
    """The oracle as it stands, timed on this host's cores on a bounded sample of the workload.  Configuration 5: whole
    tenants' stacks as a chain (activations rounded to bf16 between layers), which also gives the end-to-end drift of
    the HIP path's final activations against that chain (reported, not gated)."""
    import numpy as np
    from oracle import oracle
    from paper_1901_00041_amd import synth
    out = {"unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle"}
    if cfg == 5:
        spent = flops = layers = 0
        drift = []
        t = 0
        if wl is not None:
            # one clean lock-step pass of the headline form from the seeded inputs (the extras leave tenants mid-network)
            form = HEADLINE_FORM[5] if HEADLINE_FORM[5] in wl.forms else "fused"
            wl.run(form, None)
            wl.torch.cuda.synchronize()
        while spent < budget_s and t < synth.N_TENANTS[5]:
            ref, s, f, n = _oracle_chain(t, budget_s - spent)
            spent, flops, layers = spent + s, flops + f, layers + n
            if ref is not None and wl is not None:
                last = wl.stack.steps[-1]
                sh = last.shape
                got = wl.stack.view(last.dst, t, sh.N, sh.P, sh.Q, sh.K).double().cpu().numpy().transpose(0, 3, 1, 2)
                drift.append({"tenant": t, "max_abs_err_over_max_abs_ref": float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30)),
                              "rel_l2": float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30))})
            t += 1
        out.update({"value": flops / spent / 1e12,
                    "sample": f"configs[4]: {layers} conv layers of tenants 0..{t - 1} in stack order, {flops / 1e9:.2f} GFLOP in "
                              f"{spent:.1f} s inside the fp64 direct convolution (gcc -O2, OpenMP)"})
        if drift:
            out["end_to_end_drift"] = {"what": "final 2048x7x7 activations of the HIP path after one pass against an fp64 oracle chain that "
                                               "rounds activations to bf16 at the same points; reported, not gated", "tenants": drift}
        return out
    shapes = synth.config_shapes(cfg)
    tensors = [(synth.gen_input(cfg, t, 0, s).astype("float64"), synth.gen_weight(cfg, t, 0, s).astype("float64"), s)
               for t, s in enumerate(shapes)]
    spent = flops = n = 0
    while spent < budget_s and n < 2000:
        for x, w, s in tensors:
            t0 = time.perf_counter()
            oracle.conv2d(x, w, s.stride, s.pad)
            spent += time.perf_counter() - t0
            flops += s.flops
            n += 1
            if spent >= budget_s:
                break
    out.update({"value": flops / spent / 1e12,
                "sample": f"configs[{cfg - 1}]: {n} layer evaluations over whole tenants in order, {flops / 1e9:.2f} GFLOP in {spent:.1f} s"})
    return out


_ORACLE_LEG = r"""
import sys, time, json
sys.path.insert(0, %r)
from oracle import oracle
from paper_1901_00041_amd import synth
cfg, reps = int(sys.argv[1]), int(sys.argv[2])
ts = [(synth.gen_input(cfg, t, 0, s).astype("float64"), synth.gen_weight(cfg, t, 0, s).astype("float64"), s)
      for t, s in enumerate(synth.config_shapes(cfg))]
best = None
for _ in range(reps):
    t0 = time.perf_counter()
    for x, w, s in ts:
        oracle.conv2d(x, w, s.stride, s.pad)
    dt = time.perf_counter() - t0
    best = dt if best is None else min(best, dt)
print(json.dumps({"seconds": best, "gflops": sum(s.flops for _, _, s in ts) / best / 1e9, "threads": oracle.num_threads()}))
"""


def oracle_legs():
    """Whole configurations 1-4 through the oracle in a child process each: all host threads (three repetitions for
    configurations 1-3, one for 4) and a single thread for configurations 1-3 (OMP_NUM_THREADS=1)."""
    out = {}
    for cfg in (1, 2, 3, 4):
        for label, env in (("all_threads", {}), ("single_thread", {"OMP_NUM_THREADS": "1"})):
            if label == "single_thread" and cfg == 4:
                continue
            e = dict(os.environ)
            e.update(env)
            try:
                res = subprocess.run([sys.executable, "-c", _ORACLE_LEG % ROOT, str(cfg), "3" if cfg < 4 else "1"],
                                     capture_output=True, text=True, env=e, timeout=300)
                out.setdefault(str(cfg), {})[label] = json.loads(res.stdout.strip().splitlines()[-1])
            except Exception as ex:   # the oracle leg is a reported baseline; its failure must not hide the GPU numbers
                out.setdefault(str(cfg), {})[label] = {"error": repr(ex)}
    return out


# ----------------------------------------------------------------------------------------------------------------
# other modes
# ----------------------------------------------------------------------------------------------------------------
TABLE1_SHAPES = {"conv_resnet18 (M=256,N=128,K=1152)": (1, 128, 16, 16, 128, 3, 3, 1, 1),
                 "matvec_rnn (512,1,512)": (1, 512, 1, 1, 512, 1, 1, 1, 0),
                 "square (256,256,256)": (1, 256, 16, 16, 256, 1, 1, 1, 0)}
TABLE1_CFG_KEY = 41          # stream key of the seeded generator for these tenants (tests use the same)


def table1_tenants(shape, r, dtype):
    """R identical-shape tenants of one Table-1 problem from the seeded generator: (keep, descs)."""
    import torch
    from paper_1901_00041_amd import st_conv as sc
    from paper_1901_00041_amd import synth
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]
    N, C, H, W, K, R_, S_, st, pd = shape
    s = synth.ConvShape(N, C, H, W, K, R_, S_, st, pd, dtype, "f32")
    keep, descs = [], []
    for t in range(r):
        x = torch.from_numpy(synth.gen_input(TABLE1_CFG_KEY, t, 0, s).transpose(0, 2, 3, 1).copy()).to(tdt).cuda()
        w = torch.from_numpy(synth.gen_weight(TABLE1_CFG_KEY, t, 0, s).transpose(0, 2, 3, 1).copy()).to(tdt).cuda()
        y = torch.empty((N, s.P, s.Q, K), dtype=torch.float32, device="cuda")
        keep.append((x, w, y))
        descs.append(sc.make_desc(N, C, H, W, K, R_, S_, st, pd, dtype, "f32", x, w, y))
    return keep, descs


def paper_sweep(iters: int = 400, warmup: int = 40):
    """The paper's kernel-level experiment (Section 4.1, Figure 7, Table 1) on this GPU: R same-shape tenants, own
    weights and inputs each (seeded generator, the tensors the parity test checks), R from 2 to 120, the three problem
    shapes of Table 1 as convolutions, under the three issue policies, one batch at a time.  Speed-up of the fused
    launch over the next best policy at R = 10, R = 20 and as a geometric mean over R, fp32 and bf16."""
    import torch
    from paper_1901_00041_amd import st_conv as sc
    rs = [2, 4, 6, 8, 10, 14, 20, 28, 40, 56, 80, 120]
    streams = [torch.cuda.Stream() for _ in range(max(rs))]
    out = {}

    def timed(fn, stream):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / iters

    for dtype in ("f32", "bf16"):
        for name, shape in TABLE1_SHAPES.items():
            rows = []
            for r in rs:
                keep, descs = table1_tenants(shape, r, dtype)
                plan = sc.st_conv_plan(descs, keep=keep)
                solo = [sc.st_conv_plan([d], keep=keep) for d in descs]
                flops = int(sc.st_conv_plan_info(plan).flops)
                s0 = torch.cuda.Stream()
                use = [s0] + streams[1:r]
                t = {"fused": timed(lambda: sc.st_conv_run(plan, s0), s0),
                     "time_only_same_tiles": timed(lambda: sc.st_conv_run_time_only(plan, s0), s0),
                     "space_only_same_tiles": timed(lambda: sc.st_conv_run_space_only(plan, use), s0),
                     "time_only_retuned": timed(lambda: sc.st_conv_run_plans_time_only(solo, s0), s0),
                     "space_only_retuned": timed(lambda: sc.st_conv_run_plans_space_only(solo, use), s0)}
                t_time = min(t["time_only_same_tiles"], t["time_only_retuned"])
                t_space = min(t["space_only_same_tiles"], t["space_only_retuned"])
                rows.append({"R": r, "us": t, "fused_tflops": flops / (t["fused"] * 1e-6) / 1e12,
                             "vs_time_only": t_time / t["fused"], "vs_space_only": t_space / t["fused"],
                             "vs_next_best": min(t_time, t_space) / t["fused"],
                             "next_best": "time_only" if t_time <= t_space else "space_only"})
            print(f"paper sweep: {dtype} {name} done", file=sys.stderr, flush=True)
            gm = lambda key: math.exp(sum(math.log(x[key]) for x in rows) / len(rows))
            out[f"{dtype} {name}"] = {"rows": rows, "geomean_vs_time_only": gm("vs_time_only"),
                                      "geomean_vs_space_only": gm("vs_space_only"), "geomean_vs_next_best": gm("vs_next_best"),
                                      "R10_vs_next_best": next(x["vs_next_best"] for x in rows if x["R"] == 10),
                                      "R20_vs_next_best": next(x["vs_next_best"] for x in rows if x["R"] == 20)}
    return {"mode": "paper_sweep", "R": rs, "results": out, "inputs": "seeded generator, stream key 41 (parity: tests/test_gpu_table1.py)",
            "paper_table1_V100_fp32": {"conv": {"R10": 1.68, "R20": 2.88, "geomean": 3.23, "next_best": "space_only"},
                                       "matvec": {"R10": 1.21, "R20": 2.14, "geomean": 2.48, "next_best": "time_only"},
                                       "square": {"R10": 2.42, "R20": 2.47, "geomean": 4.93, "next_best": "space_only"},
                                       "conv_geomean_vs_time_only": [7.73, 7.71]}}


def arrival_trace(steps: int = 400, p_ready: float = 0.7, capacity: int = 256, seed: int = 11):
    """Dynamic arrival (Section 4: the scheduler merges whichever kernels are ready and caches the merged kernels): a
    pool of 8 tenants (configs[1]'s four layers and four of configs[2]'s), a seeded Bernoulli ready set per step,
    plans from the plan cache.  Host time of the cache call (hit / miss), hit rate, and the whole trace's
    throughput against launching every ready tenant on its own (time-only, per-tenant plans).  Timing only: tensors
    come from torch's generator."""
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
    cache.destroy()
    return out


def isolation(reps: int = 30):
    """Predictability (Section 3: identical models sharing a GPU under spatial multiplexing finish up to 25% apart): R
    identical tenants (the Section 4.1 convolution, own weights and inputs each); per-tenant completion time inside
    one fused launch (in-kernel clock) and under the space-only policy (one stream per tenant, HIP events).
    gap = (slowest - fastest) / slowest over the tenants' mean completion times.  Timing only."""
    import numpy as np
    import torch
    from paper_1901_00041_amd import st_conv as sc
    out = {"mode": "isolation", "shape": "3x3 128->128 @16x16 (M=256, N=128, K=1152), bf16 in / fp32 out", "results": {}}
    for R in (8, 32):
        keep, descs = table1_tenants(TABLE1_SHAPES["conv_resnet18 (M=256,N=128,K=1152)"], R, "bf16")
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


def occupancy(cfg: int, reps: int = 5):
    """Occupancy per tenant inside one fused launch, from the in-kernel time stamps of st_conv_run_profiled: per tenant
    its work items, the workgroup-time they were resident for (sum of item durations), its share of the launch's
    total workgroup-time, the mean number of its workgroups resident over the launch, and its first start and last
    end.  Prints a markdown table (median over `reps` launches)."""
    import numpy as np
    import torch
    from paper_1901_00041_amd import st_conv as sc
    wl = Workload(cfg)
    items = sc.st_conv_plan_worklist(wl.plan, 0)
    n_t = len(wl.shapes)
    for _ in range(3):
        sc.st_conv_run(wl.plan)
    torch.cuda.synchronize()
    rows = []
    for _ in range(reps):
        st = sc.st_conv_run_profiled(wl.plan).astype(np.int64)
        t0 = st[:, 4].min()
        b, e = (st[:, 4] - t0) * 10.0, (st[:, 6] - t0) * 10.0         # ns, 100 MHz clock
        total = float(e.max())
        per = []
        for t in range(n_t):
            m = items["tenant"] == t
            per.append((int(m.sum()), float((e[m] - b[m]).sum()), float(b[m].min()), float(e[m].max()), total))
        rows.append(per)
    med = np.median(np.array(rows), axis=0)
    wg_time = med[:, 1].sum()
    lines = [f"| tenant | layer (M x N x K) | tile | split-K | work items | resident workgroup-time (us) | share of launch | mean workgroups resident | first start (us) | last end (us) |",
             "|---|---|---|---|---|---|---|---|---|---|"]
    for t in range(n_t):
        ti = sc.st_conv_plan_tenant_info(wl.plan, t)
        n, busy, first, last, total = med[t]
        lines.append(f"| {t} | {ti.M} x {ti.Ngemm} x {ti.Kgemm} | {ti.MT}x{ti.NT} | {ti.split_k} | {int(n)} | {busy / 1e3:.1f} | "
                     f"{100 * busy / wg_time:.1f} % | {busy / total:.1f} | {first / 1e3:.2f} | {last / 1e3:.2f} |")
    total = float(med[0, 4])
    lines.append("")
    lines.append(f"Launch: {int(med[:, 0].sum())} work items, {total / 1e3:.2f} us from the first workgroup's start to the last one's end, "
                 f"{wg_time / total:.1f} workgroups resident on average (512 slots: two per compute unit).")
    return "\n".join(lines)


def probes():
    """What this chip reaches on a plain copy and on a register-only MFMA loop (libst_bench_probe.so, a bench helper
    outside the convolution library), beside the published peaks the roofline is priced against."""
    import ctypes
    path = os.path.join(ROOT, "paper_1901_00041_amd", "libst_bench_probe.so")
    if not os.path.exists(path):
        return None
    L = ctypes.CDLL(path)
    L.st_bench_probe_chip.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    vals = []
    for what in range(4):
        r = ctypes.c_double()
        if L.st_bench_probe_chip(what, ctypes.byref(r)) != 0:
            return None
        vals.append(r.value)
    return {"hbm_copy_GBps": vals[0] / 1e9, "mfma_bf16_TFLOPs": vals[1] / 1e12, "mfma_f16_TFLOPs": vals[2] / 1e12,
            "mfma_f32_TFLOPs": vals[3] / 1e12,
            "published": {"hbm_GBps": PEAK_HBM_GBS, "mfma_bf16_TFLOPs": PEAK_BF16_TFLOPS, "mfma_f32_TFLOPs": PEAK_F32_TFLOPS}}


# ----------------------------------------------------------------------------------------------------------------
def measure(cfg: int, steps: int, warmup: int, policies, extras: bool, extra_steps: int = 4):
    passes = PASSES_PER_STEP[cfg]
    copies = 1
    if extras and cfg != 5:
        # enough copies of the tensors to exceed the 256 MB memory-side cache several times over (cold-cache extra)
        copies = min(160, max(4, int(1.2e9 // {1: 475e3, 2: 8.52e6, 3: 14.25e6, 4: 104.4e6}[cfg])))
    wl = Workload(cfg, copies)
    head = HEADLINE_FORM[cfg] if HEADLINE_FORM[cfg] in wl.forms else "fused"
    out = {"flops": wl.flops, "algorithmic_bytes": wl.bytes, "plan_build_us": round(wl.plan_build_us, 1),
           "work_items": wl.n_items, "passes_per_step": passes, "steps": steps, "headline_form": head, "policies": {}}
    for form in wl.forms:
        if policies and form not in policies and form != head:
            continue
        out["policies"][form] = time_form(wl, form, steps, warmup, passes)
        print(f"bench: config {cfg} {form}: {out['policies'][form]['us_per_pass']:.2f} us per pass", file=sys.stderr, flush=True)
    pol = out["policies"]
    fused = pol[head]
    out["value_tflops"] = fused["tflops"]
    out["pct_bf16_mfma_peak"] = 100.0 * fused["tflops"] / PEAK_BF16_TFLOPS
    for base in ("time_only", "space_only"):
        cands = {f: pol[f]["ms_per_step"] for f in (base, base + "_retuned") if f in pol}
        if cands:
            best = min(cands, key=cands.get)
            out[f"speedup_vs_{base}"] = cands[best] / fused["ms_per_step"]
            out[f"{base}_form"] = best
    out["roofline"] = roofline(wl, head, fused)
    out["rooflines"] = {f: roofline(wl, f, pol[f]) for f in pol if f in wl.launches}
    if extras:
        ex = {}
        for form in wl.extra_forms:
            try:
                if cfg != 5 and form in PIPELINED:
                    ex[form] = time_pipelined_native(wl, form, extra_steps, 1, passes)
                elif form == "space_only_free":
                    ex[form] = time_free_running(wl, extra_steps, 1, passes)
                else:
                    ppr = getattr(wl, "passes_per_run", {}).get(form, 1)
                    r = time_form(wl, form, extra_steps, 1, max(1, passes // (4 if cfg == 5 else 1) // ppr))
                    ex[form] = {"us_per_pass": r["us_per_pass"] / ppr, "tflops": r["tflops"] * ppr, "timed_region_s": r["timed_region_s"]}
            except Exception as e:      # an extra that cannot run is reported; it does not enter `value`
                ex[form] = {"error": repr(e)}
            print(f"bench: config {cfg} extra {form}: {ex[form]}", file=sys.stderr, flush=True)
        out["extras"] = ex
    return out, wl


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=HEADLINE_CONFIG, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--no-sweep", action="store_true", help="skip the other configurations")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-extras", action="store_true", help="skip the forms that do not enter `value` (several batches in flight, "
                    "free-running streams, cold caches, staggered tenants)")
    ap.add_argument("--policies", default="", help="comma-separated forms to time (default: all); the headline form always runs")
    ap.add_argument("--paper-sweep", action="store_true", help="the paper's R-sweep of its three Table-1 shapes")
    ap.add_argument("--arrival-trace", action="store_true", help="a synthetic trace whose ready set changes every step, through the plan cache")
    ap.add_argument("--isolation", action="store_true", help="per-tenant completion spread of identical tenants: fused launch vs space-only")
    ap.add_argument("--occupancy", action="store_true", help="per-tenant occupancy table of one fused launch of --config (1-4), as markdown")
    ap.add_argument("--probes", action="store_true", help="achievable copy bandwidth and MFMA rates of this chip")
    ap.add_argument("--form", default="", help="with --counters: the form to run (default: the headline form of --config)")
    ap.add_argument("--counters", action="store_true",
                    help="counter-collection mode for rocprofv3 --pmc: only K passes of the headline form of --config and K launches "
                         "of a 64 MiB copy kernel (the known-traffic reference); prints a short JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (tenants are independent; sharding is placement only). "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1901_00041_amd import st_conv as sc
    from paper_1901_00041_amd import synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    sc.lib()
    torch.cuda.set_device(0)

    if args.paper_sweep:
        print(json.dumps(paper_sweep()))
        return
    if args.arrival_trace:
        print(json.dumps(arrival_trace()))
        return
    if args.isolation:
        print(json.dumps(isolation()))
        return
    if args.occupancy:
        print(occupancy(args.config))
        return
    if args.probes:
        print(json.dumps({"mode": "probes", "chip": probes()}))
        return
    if args.counters:
        wl = Workload(args.config)
        form = args.form or HEADLINE_FORM[args.config]
        k = args.steps
        src = torch.empty(64 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(k):
            wl.run(form, None)
        for _ in range(k):
            sc.st_launch_copy(src, dst, src.numel(), None)
        torch.cuda.synchronize()
        print(json.dumps({"mode": "counters", "workload": CONFIG_TEXT[args.config], "form": form, "passes": k,
                          "launches_per_pass": wl.launches.get(form, 1), "algorithmic_bytes_per_pass": wl.bytes, "flops_per_pass": wl.flops,
                          "copy_launches": k, "copy_bytes_read": src.numel(), "copy_bytes_written": src.numel()}))
        return

    policies = [p for p in args.policies.split(",") if p]
    floor_us = launch_floor_us()
    head, wl = measure(args.config, args.steps, args.warmup, policies, not args.no_extras)
    form = head["headline_form"]
    fused = head["policies"][form]
    line = {
        "metric": "aggregate conv TFLOP/s (% bf16 MFMA peak) + speedup vs time-only/space-only",
        "value": fused["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": fused["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if args.config == 1 else "bf16", "data": "synthetic",
        "config": {"workload": CONFIG_TEXT[args.config], "policy": POLICY_TEXT.get(form, form), "form": form,
                   "tenants": synth.N_TENANTS[args.config], "passes_per_step": head["passes_per_step"],
                   "us_per_pass": fused["us_per_pass"], "flops_per_pass": head["flops"]},
        "event_ms_per_step": fused["event_ms_per_step"], "timed_region_s": fused["timed_region_s"],
        "pct_bf16_mfma_peak": head["pct_bf16_mfma_peak"],
        "speedup_vs_time_only": head.get("speedup_vs_time_only"), "speedup_vs_space_only": head.get("speedup_vs_space_only"),
        "baseline_forms": {"time_only": head.get("time_only_form"), "space_only": head.get("space_only_form")},
        "policies": head["policies"],
        "launch_floor_us": floor_us, "plan_build_us": head["plan_build_us"], "work_items": head["work_items"],
        "gpu_max_hw_queues": os.environ.get("GPU_MAX_HW_QUEUES", "default(4)"),
        "roofline": head["roofline"],
        "paper_context": PAPER_CONTEXT,
    }
    line["rooflines"] = head["rooflines"]
    if "extras" in head:
        line["extras"] = head["extras"]
    if not args.no_extras:
        line["roofline"]["achievable"] = probes()
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(args.config, wl)
    del wl
    failed = []
    if not args.no_sweep:
        per_config = {}
        for cfg in (1, 2, 3, 4, 5):
            if cfg == args.config:
                per_config[str(cfg)] = {k: v for k, v in head.items()}
                continue
            try:
                r, w = measure(cfg, max(5, args.steps // 2), 2, policies, not args.no_extras)
                del w
                per_config[str(cfg)] = r
            except Exception as e:      # reported, and the run fails below
                per_config[str(cfg)] = {"error": repr(e)}
                failed.append(cfg)
        ok = [v for v in per_config.values() if "error" not in v]
        for base in ("time_only", "space_only"):
            vals = [v[f"speedup_vs_{base}"] for v in ok if f"speedup_vs_{base}" in v]
            if vals:
                per_config[f"geomean_speedup_vs_{base}"] = math.exp(sum(math.log(x) for x in vals) / len(vals))
        line["per_config"] = per_config
        if not args.no_cpu:
            line["cpu_baseline"]["whole_configs"] = oracle_legs()
    print(json.dumps(line))
    if failed:
        print(f"bench.py: configurations {failed} failed", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
