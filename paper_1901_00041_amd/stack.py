"""Configuration 5: several tenants, each running a ResNet-50-shaped stack of 53 convolution layers,
scheduled layer by layer: step s of every tenant goes into one fused launch (one cached plan per step).
Consecutive steps that do not depend on each other (a block's projection conv and its first 1x1 conv both
read the block input) are co-scheduled: the fused policy issues them as one launch over both steps'
descriptors.  A second schedule keeps the tenants at DIFFERENT depths of the network (requests that arrived
at different times): every fused launch then mixes as many different layer shapes as there are tenants (the heterogeneous
case that the paper's application model, Section 2, sets aside as future work).

Data flow per tenant (no batch-norm): stem conv + ReLU, 3x3/2 max-pool, then per bottleneck
a = ReLU(conv1(x)), b = ReLU(conv2(a)), out = ReLU(conv3(b) + shortcut), shortcut = x or proj(x).
Activations are stored as bf16; the residual add and the ReLU run in the conv epilogue on the fp32
accumulator.  All arithmetic runs in the library's kernels; this module only allocates device memory,
builds the descriptors and issues the run calls.
"""
from __future__ import annotations

import time
from typing import List

import numpy as np

from . import st_conv as sc
from . import synth


# Workgroup slots the planner fills per launch when the caller gives no options.  Every launch of the stack is followed
# by one that depends on it, so a launch's slowest work item and its tail count for more than in a launch that stands
# alone, and somewhat fewer, larger work items than the planner's default (400) do better: measured per pass of 8
# tenants, 200 slots 560 us, 250 555, 300 545, 350 572, 400 578, 450 581.
STACK_SLOTS = 300


class ResNetStack:
    def __init__(self, n_tenants: int = 8, cfg: int = 5, batch: int = 1, image: int = 224, seeded_weights: bool = True,
                 plan_opts=None, co_schedule: bool = True, unique_buffers: bool = False):
        import torch
        self.torch = torch
        if plan_opts is None:
            plan_opts = sc.plan_opts(target_items=STACK_SLOTS)
        self.n_tenants, self.cfg = n_tenants, cfg
        self.steps: List[synth.Step] = synth.resnet50_steps(batch, image)
        if unique_buffers:
            # every step writes a buffer of its own (nothing is overwritten within a pass), so that after ONE launch
            # over the whole network every layer's inputs and outputs can still be read back
            import dataclasses
            latest, fresh, steps = {0: 0}, 100, []
            for st in self.steps:
                src, res = latest[st.src], (latest[st.res] if st.res is not None else None)
                dst, fresh = fresh, fresh + 1
                pool_dst = None
                if st.pool_after:
                    pool_dst, fresh = fresh, fresh + 1
                steps.append(dataclasses.replace(st, src=src, dst=dst, res=res, pool_dst=pool_dst))
                latest[st.dst] = dst
                if st.pool_after:
                    latest[st.pool_dst] = pool_dst
            self.steps = steps
        dev = "cuda"
        # activation buffers: one tensor per buffer id holding every tenant (tenant-major), sized for the
        # largest use of that id
        need = {}
        for st in self.steps:
            s = st.shape
            need[st.src] = max(need.get(st.src, 0), s.N * s.H * s.W * s.C)
            need[st.dst] = max(need.get(st.dst, 0), s.N * s.P * s.Q * s.K)
            if st.pool_after:
                p = (s.P + 2 - 3) // 2 + 1
                need[st.pool_dst] = max(need.get(st.pool_dst, 0), s.N * p * p * s.K)
        self.buf = {i: torch.zeros((n_tenants, n), dtype=torch.bfloat16, device=dev) for i, n in need.items()}
        # network inputs and weights from the seeded generator
        s0 = self.steps[0].shape
        for t in range(n_tenants):
            x = synth.gen_input(cfg, t, 0, s0)
            self.buf[0][t, :x.size] = torch.from_numpy(np.ascontiguousarray(x.transpose(0, 2, 3, 1)).reshape(-1)).to(torch.bfloat16)
        self.weights = []          # [step][tenant] device tensors, KRSC
        for st in self.steps:
            s, row = st.shape, []
            for t in range(n_tenants):
                if seeded_weights:
                    w = synth.gen_weight(cfg, t, st.index, s, 2.0)
                    row.append(torch.from_numpy(np.ascontiguousarray(w.transpose(0, 2, 3, 1))).to(torch.bfloat16).to(dev))
                else:
                    g = torch.Generator(device=dev).manual_seed(1000 * st.index + t)
                    row.append((torch.randn((s.K, s.R, s.S, s.C), device=dev, generator=g) *
                                (2.0 / (s.C * s.R * s.S)) ** 0.5).to(torch.bfloat16))
            self.weights.append(row)
        # one plan per step
        self.plans, t_plan = [], []
        self.flops = self.bytes = self.n_items = 0
        step_descs = []
        for st in self.steps:
            s = st.shape
            epi = (sc.ST_EPI_RELU if st.relu else 0) | (sc.ST_EPI_RESIDUAL if st.res is not None else 0)
            descs = [sc.make_desc(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, "bf16", "bf16",
                                  self.buf[st.src][t], self.weights[st.index][t], self.buf[st.dst][t],
                                  self.buf[st.res][t] if st.res is not None else None, epi)
                     for t in range(n_tenants)]
            step_descs.append(descs)
            t0 = time.perf_counter()
            plan = sc.st_conv_plan(descs, plan_opts)
            t_plan.append((time.perf_counter() - t0) * 1e6)
            self.plans.append(plan)
            info = sc.st_conv_plan_info(plan)
            self.flops += int(info.flops)
            self.bytes += int(info.bytes)
            self.n_items += int(info.n_items)
        self.plan_build_us = float(np.median(t_plan))
        # groups of consecutive, mutually independent steps; each group of more than one step gets a plan of
        # its own over all its descriptors
        self.groups: List[List[int]] = []
        for st in self.steps:
            if co_schedule and self.groups and self._independent(self.groups[-1], st):
                self.groups[-1].append(st.index)
            else:
                self.groups.append([st.index])
        self.group_plans = []
        for g in self.groups:
            if len(g) == 1:
                self.group_plans.append(self.plans[g[0]])
            else:
                self.group_plans.append(sc.st_conv_plan([d for i in g for d in step_descs[i]], plan_opts))
        self.n_items = sum(int(sc.st_conv_plan_info(p).n_items) for p in self.group_plans)
        self.n_launches = len(self.groups)
        self._step_descs = step_descs
        self._plan_opts = plan_opts
        self._solo = None          # [step][tenant] plans of one tenant each, built on first use
        self._streams = [torch.cuda.Stream() for _ in range(n_tenants)]

    def _independent(self, group: List[int], st) -> bool:
        """True when step `st` neither reads what a step of the group writes nor writes what one reads or writes."""
        for i in group:
            g = self.steps[i]
            if g.pool_after or st.pool_after:
                return False
            if st.src in (g.dst,) or (st.res is not None and st.res == g.dst):
                return False
            if st.dst in (g.src, g.dst) or (g.res is not None and st.dst == g.res):
                return False
        return True

    # ---- execution -----------------------------------------------------------------------------------
    def run_group(self, gi: int, stream=None) -> None:
        """One fused launch over every tenant's descriptors of every step of group gi."""
        sc.st_conv_run(self.group_plans[gi], stream)
        for i in self.groups[gi]:
            st = self.steps[i]
            if st.pool_after:
                s = st.shape
                sc.st_maxpool_nhwc(self.buf[st.dst], self.buf[st.pool_dst], self.n_tenants * s.N, s.P, s.Q, s.K, 3, 2, 1,
                                   "bf16", stream)

    def solo_plans(self, i: int):
        """Step i's tenants planned one by one: the baselines' tiles when every launch has the GPU to itself."""
        if self._solo is None:
            self._solo = [[sc.st_conv_plan([d], self._plan_opts) for d in descs] for descs in self._step_descs]
        return self._solo[i]

    def run_step(self, i: int, policy: str = "fused", stream=None) -> None:
        st = self.steps[i]
        if policy == "fused":
            sc.st_conv_run(self.plans[i], stream)
        elif policy == "time_only":
            sc.st_conv_run_time_only(self.plans[i], stream)
        elif policy == "space_only":
            sc.st_conv_run_space_only(self.plans[i], [stream] + self._streams[1:])
        elif policy == "time_only_retuned":
            sc.st_conv_run_plans_time_only(self.solo_plans(i), stream)
        elif policy == "space_only_retuned":
            sc.st_conv_run_plans_space_only(self.solo_plans(i), [stream] + self._streams[1:])
        else:
            raise ValueError(f"unknown policy {policy!r}")
        if st.pool_after:
            s = st.shape
            # all tenants' stem outputs are one contiguous batch: a single pooling launch
            sc.st_maxpool_nhwc(self.buf[st.dst], self.buf[st.pool_dst], self.n_tenants * s.N, s.P, s.Q, s.K, 3, 2, 1,
                               "bf16", stream)

    def run_chains(self, stream=None) -> None:
        """Space-only without per-layer joins: every tenant's whole chain of per-tenant launches goes to the tenant's
        own stream; the streams fork from `stream` at the start and join it at the end."""
        torch = self.torch
        anchor = stream if stream is not None else torch.cuda.current_stream()
        start = torch.cuda.Event()
        start.record(anchor)
        streams = [anchor] + self._streams[1:]
        for s in streams[1:]:
            s.wait_event(start)
        # runs of steps without pooling go to the library's issue loop in one call (tenant t on stream t; the loop
        # issues from several host threads, which this many small launches need: 424 per pass)
        run: list = []
        for i, st in enumerate(self.steps):
            run.extend(self.solo_plans(i))
            if st.pool_after or i == len(self.steps) - 1:
                sc.st_conv_run_plans_on_streams_many(run, streams, 1)
                run = []
            if st.pool_after:
                s = st.shape
                for t in range(self.n_tenants):
                    sc.st_maxpool_nhwc(self.buf[st.dst][t], self.buf[st.pool_dst][t], s.N, s.P, s.Q, s.K, 3, 2, 1, "bf16",
                                       streams[t])
        for s in streams[1:]:
            done = torch.cuda.Event()
            done.record(s)
            anchor.wait_event(done)

    # ---- tenants at different depths ---------------------------------------------------------------
    def staggered_groups(self, g: int):
        """[(tenant, group index)] of global step g in the staggered schedule: tenant t runs group
        (g + offset_t) mod n_groups, i.e. the tenants sit at different depths of the network and every tenant
        still walks its own layers in order (wrapping from the last layer to the first of its next image)."""
        G = len(self.groups)
        return [(t, (g + self.stagger_offsets[t]) % G) for t in range(self.n_tenants)]

    def build_staggered(self, offsets=None) -> None:
        """Plans for the steady state of a server whose tenants' requests arrived at different times: one fused
        launch per global step over every tenant's CURRENT group of layers, which differ in shape from tenant to
        tenant.  offsets default to an even spread over the depth of the network."""
        G = len(self.groups)
        self.stagger_offsets = list(offsets) if offsets is not None else [(t * G) // self.n_tenants for t in range(self.n_tenants)]
        assert len(self.stagger_offsets) == self.n_tenants
        self.staggered_plans = []
        for g in range(G):
            descs = [self._step_descs[i][t] for t, gi in self.staggered_groups(g) for i in self.groups[gi]]
            self.staggered_plans.append(sc.st_conv_plan(descs, self._plan_opts))
        self.n_items_staggered = sum(int(sc.st_conv_plan_info(p).n_items) for p in self.staggered_plans)

    def run_staggered_step(self, g: int, stream=None, policy: str = "fused") -> None:
        """Global step g of the staggered schedule (build_staggered first): one fused launch, or the same work
        items as one launch per tenant-layer on one stream (time_only) or on one stream each (space_only)."""
        if policy == "fused":
            sc.st_conv_run(self.staggered_plans[g], stream)
        elif policy == "time_only":
            sc.st_conv_run_time_only(self.staggered_plans[g], stream)
        elif policy == "space_only":
            sc.st_conv_run_space_only(self.staggered_plans[g], [stream] + self._streams[1:])
        else:
            raise ValueError(f"unknown policy {policy!r}")
        for t, gi in self.staggered_groups(g):
            for i in self.groups[gi]:
                st = self.steps[i]
                if st.pool_after:
                    s = st.shape
                    sc.st_maxpool_nhwc(self.buf[st.dst][t], self.buf[st.pool_dst][t], s.N, s.P, s.Q, s.K, 3, 2, 1, "bf16",
                                       stream)

    # ---- tenant groups: fused launches per group, groups side by side ---------------------------------
    def build_tenant_groups(self, n_groups: int, opts=None) -> None:
        """Split the tenants into n_groups groups of consecutive tenants.  Every group gets its own chain of fused
        launches (one per layer group, over the group's tenants only), planned for its share of the GPU, and its own
        stream: within a group the tenants advance in lock-step through one launch per layer, while the groups run
        side by side and need not wait for each other's slowest tile between layers.  n_groups = 1 is the plain
        fused policy, n_groups = n_tenants the chains form of space-only."""
        assert 1 <= n_groups <= self.n_tenants
        slots = {1: 0, 2: 256, 4: 128}.get(n_groups, max(32, 512 // n_groups))       # workgroup slots a launch is planned for
        opts = opts if opts is not None else sc.plan_opts(target_items=slots)
        bounds = [(g * self.n_tenants) // n_groups for g in range(n_groups + 1)]
        self.tenant_groups = [list(range(bounds[g], bounds[g + 1])) for g in range(n_groups)]
        self.tenant_group_plans = [[sc.st_conv_plan([self._step_descs[i][t] for i in lg for t in tg], opts)
                                    for lg in self.groups] for tg in self.tenant_groups]

    def run_tenant_groups(self, stream=None) -> None:
        """One pass: every tenant group's chain of fused launches on its own stream; the streams fork from `stream`
        at the start and join it at the end (build_tenant_groups first)."""
        torch = self.torch
        anchor = stream if stream is not None else torch.cuda.current_stream()
        streams = [anchor] + self._streams[1:len(self.tenant_groups)]
        start = torch.cuda.Event()
        start.record(anchor)
        for s in streams[1:]:
            s.wait_event(start)
        # issue layer by layer, round-robin over the groups, so that no stream's queue runs dry while another's fills
        for gi, lg in enumerate(self.groups):
            for g, tg in enumerate(self.tenant_groups):
                sc.st_conv_run(self.tenant_group_plans[g][gi], streams[g])
                for i in lg:
                    st = self.steps[i]
                    if st.pool_after:
                        s = st.shape
                        sc.st_maxpool_nhwc(self.buf[st.dst][tg[0]:tg[-1] + 1], self.buf[st.pool_dst][tg[0]:tg[-1] + 1],
                                           len(tg) * s.N, s.P, s.Q, s.K, 3, 2, 1, "bf16", streams[g])
        for s in streams[1:]:
            done = torch.cuda.Event()
            done.record(s)
            anchor.wait_event(done)

    # ---- the whole pass as one persistent launch --------------------------------------------------------
    def build_chain(self, chain_queues: int = 0) -> None:
        """One chain over every tenant's whole network: tenant t is sequence t; a layer group is a stage (the
        projection conv and the block's first 1x1 conv share one), the max-pool after the stem a stage of its own.
        Planned with the stack's own options, so every stage gets the tiles of the layer-by-layer plans."""
        po = self._plan_opts
        opts = sc.plan_opts(tile_cfg=po.tile_cfg, split_k=po.split_k, target_items=po.target_items,
                            rows_per_tile=po.rows_per_tile, chain_queues=chain_queues)
        ops = []
        for gi, group in enumerate(self.groups):
            for i in group:
                st = self.steps[i]
                s = st.shape
                for t in range(self.n_tenants):
                    ops.append(sc.make_chain_op(sc.ST_OP_CONV, t, 2 * gi, self._step_descs[i][t]))
                    if st.pool_after:
                        p = (s.P + 2 - 3) // 2 + 1
                        d = sc.make_desc(s.N, s.K, s.P, s.Q, s.K, 3, 3, 2, 1, "bf16", "bf16", self.buf[st.dst][t], None, self.buf[st.pool_dst][t])
                        ops.append(sc.make_chain_op(sc.ST_OP_MAXPOOL, t, 2 * gi + 1, d))
        self.chain = sc.Chain(ops, opts, keep=[self.buf, self.weights])
        self.chain_ops = ops

    def run(self, policy: str = "fused", stream=None) -> None:
        if policy == "fused_chain":
            if getattr(self, "chain", None) is None:
                self.build_chain()
            self.chain.run(stream)
            return
        if policy.startswith("fused_groups"):
            n = int(policy[len("fused_groups"):])
            if getattr(self, "tenant_groups", None) is None or len(self.tenant_groups) != n:
                self.build_tenant_groups(n)
            self.run_tenant_groups(stream)
            return
        if policy == "fused":
            for gi in range(len(self.groups)):
                self.run_group(gi, stream)
            return
        if policy.endswith("_staggered"):
            # one cycle: every tenant advances through all its groups once, so the work equals one lock-step pass
            if not hasattr(self, "staggered_plans"):
                self.build_staggered()
            for g in range(len(self.groups)):
                self.run_staggered_step(g, stream, policy[: -len("_staggered")])
            return
        if policy == "space_only_chains":
            self.run_chains(stream)
            return
        for i in range(len(self.steps)):
            self.run_step(i, policy, stream)

    # ---- access for tests ----------------------------------------------------------------------------
    def view(self, buf_id: int, tenant: int, n: int, h: int, w: int, c: int):
        """NHWC view of a tenant's buffer holding an (n,h,w,c) tensor."""
        return self.buf[buf_id][tenant, : n * h * w * c].view(n, h, w, c)
