"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest

from paper_1901_00041_amd import st_conv as sc
from paper_1901_00041_amd import synth
from paper_1901_00041_amd.synth import ConvShape

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    sc.lib()   # fails loudly when the HIP library was not built
    return torch


def _sync(torch):
    torch.cuda.synchronize()


# several tiles plus ragged tails in M (198 pixels), N (40 filters) and K (144, 400, 147 ...)
SMALL = [
    ConvShape(2, 16, 9, 11, 40, 3, 3, 1, 1, "bf16", "f32"),
    ConvShape(1, 32, 12, 10, 72, 3, 3, 2, 1, "bf16", "f32"),
    ConvShape(3, 64, 7, 7, 136, 1, 1, 1, 0, "bf16", "f32"),
    ConvShape(1, 16, 13, 13, 24, 5, 5, 1, 2, "bf16", "f32"),
    ConvShape(2, 8, 10, 9, 16, 3, 2, 1, 0, "bf16", "f32"),
    ConvShape(1, 3, 30, 26, 64, 7, 7, 2, 3, "bf16", "f32"),     # C=3: element-wise gather
    ConvShape(1, 24, 8, 8, 20, 3, 3, 1, 1, "f16", "f32"),
    ConvShape(2, 12, 9, 9, 36, 3, 3, 1, 1, "f32", "f32"),
    ConvShape(1, 5, 8, 9, 7, 3, 3, 2, 2, "f32", "f32"),          # odd everything, scalar stores
    ConvShape(1, 40, 6, 6, 30, 1, 1, 2, 0, "bf16", "bf16"),
    ConvShape(2, 3, 20, 32, 40, 7, 7, 2, 3, "bf16", "f32"),     # row tile (few channels), ragged filters
    ConvShape(1, 3, 9, 272, 72, 7, 7, 2, 3, "bf16", "bf16"),    # row tile, two pixel tiles per output row
    ConvShape(1, 4, 9, 16, 24, 3, 7, 1, 3, "f16", "f32"),       # row tile, stride 1, C = 4
    ConvShape(1, 96, 9, 9, 40, 3, 3, 1, 1, "bf16", "f32"),      # K = 864: seven 256-byte steps, so the two smallest
    ConvShape(1, 48, 6, 6, 24, 3, 3, 1, 1, "f32", "f32"),       #   tiles split K across wavefronts (bf16 and fp32)
]


def _run_small(torch, helpers, **opts):
    tenants = [helpers.Tenant(s, synth.gen_input(90, t, 0, s), synth.gen_weight(90, t, 0, s)) for t, s in enumerate(SMALL)]
    plan = helpers.plan_for(tenants, **opts)
    sc.st_conv_run(plan)
    _sync(torch)
    for i, t in enumerate(tenants):
        helpers.check_tenant(t, f"small[{i}] {t.shape} opts={opts}")
    return tenants, plan


@pytest.mark.parametrize("tile_cfg", [1, 2, 3, 4, 5, 6, 7])
@pytest.mark.parametrize("split_k", [1, 3])
def test_every_tile_shape_and_split(torch, tile_cfg, split_k):
    from tests import helpers
    _run_small(torch, helpers, tile_cfg=tile_cfg, split_k=split_k)


# Row tile (few input channels): every combination of how the row data sits against the 16-byte vectors of its
# LDS copy (left padding of 0, 6, 8, 18, 24 bytes), of how a filter row of S*C elements ends inside its last
# vector (S*C = 9, 10, 16, 21, 28, 30), ragged filter counts, filters taller than the 7 rows one round stages,
# images wider than one round of row vectors, one and several pixel segments per output row.
ROW_SHAPES = [
    ConvShape(1, 4, 10, 24, 64, 2, 4, 1, 2, "bf16", "f32"),      # S*C = 16, left padding 16 bytes: no shifts at all
    ConvShape(2, 3, 11, 40, 40, 3, 3, 2, 1, "bf16", "f32"),      # S*C = 9, padding 6 bytes, stride 2
    ConvShape(1, 2, 12, 36, 70, 5, 5, 1, 2, "f16", "f32"),       # S*C = 10, padding 8 bytes, two filter tiles
    ConvShape(1, 6, 9, 20, 16, 3, 5, 1, 2, "bf16", "bf16"),      # S*C = 30, padding 24 bytes
    ConvShape(1, 3, 14, 16, 64, 9, 3, 2, 1, "bf16", "f32"),      # 9 filter rows: more than one staging round
    ConvShape(1, 3, 33, 272, 64, 7, 7, 2, 3, "bf16", "f32"),     # wide image: more than one round of row vectors
    ConvShape(3, 4, 8, 8, 9, 3, 7, 1, 0, "f16", "f16"),          # S*C = 28, no padding, 9 filters
    ConvShape(1, 3, 224, 224, 64, 7, 7, 2, 3, "bf16", "bf16"),   # the ResNet stem itself
]


@pytest.mark.parametrize("rows_per_tile", [1, 2, 4])
def test_row_tile_alignments(torch, rows_per_tile):
    from tests import helpers
    tenants = [helpers.Tenant(s, synth.gen_input(91, t, 0, s), synth.gen_weight(91, t, 0, s)) for t, s in enumerate(ROW_SHAPES)]
    plan = helpers.plan_for(tenants, tile_cfg=7, rows_per_tile=rows_per_tile)
    for t in range(len(tenants)):
        ti = sc.st_conv_plan_tenant_info(plan, t)
        assert ti.row_tiled == 1 and ti.rows_per_tile == rows_per_tile, f"tenant {t} did not take the row tile"
    sc.st_conv_run(plan)
    _sync(torch)
    for i, t in enumerate(tenants):
        helpers.check_tenant(t, f"row[{i}] {t.shape} rows_per_tile={rows_per_tile}")


def test_auto_plan_small(torch):
    from tests import helpers
    _run_small(torch, helpers)


def test_equal_progress_order_and_tenant_times(torch):
    """order = 2 interleaves the tenants; results do not depend on the order of the work list.  The per-tenant
    timing call reports, for every tenant, a start inside the launch and an end after it."""
    from tests import helpers
    tenants, plan = _run_small(torch, helpers, order=2)
    first, last = sc.st_conv_run_tenant_times(plan)
    assert len(first) == len(tenants) and (first >= 0).all() and (last > first).all()
    assert first.min() == 0 and last.max() < 1_000_000        # the launch takes far less than a millisecond
    for i, t in enumerate(tenants):
        helpers.check_tenant(t, f"small[{i}] after the timed launch")


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_config_parity_all_policies(torch, cfg):
    """Full-size configurations 1-4, element by element, under the three issue policies; the three
    policies must agree bit for bit (same tiles, same summation order)."""
    from tests import helpers
    tenants = helpers.make_tenants(cfg)
    plan = helpers.plan_for(tenants)
    sc.st_conv_run(plan)
    _sync(torch)
    worst = max(helpers.check_tenant(t, f"cfg{cfg} tenant {i} fused") for i, t in enumerate(tenants))
    print(f"cfg{cfg}: max |gpu-oracle| = {worst:.3e}")
    fused = [t.dy.clone() for t in tenants]
    for t in tenants:
        t.clear()
    sc.st_conv_run_time_only(plan)
    _sync(torch)
    for i, t in enumerate(tenants):
        assert torch.equal(t.dy, fused[i]), f"time-only differs from fused for tenant {i}"
        t.clear()
    streams = [torch.cuda.Stream() for _ in tenants]
    sc.st_conv_run_space_only(plan, streams)
    _sync(torch)
    for i, t in enumerate(tenants):
        assert torch.equal(t.dy, fused[i]), f"space-only differs from fused for tenant {i}"


def test_fused_equals_solo_bitwise_and_distinct_weights(torch):
    """No cross-tenant interaction (Section 4: disjoint graphs): a tenant's fused result equals its result
    when planned alone with the same tile shape and split; tenants with equal shapes but different weights
    give different outputs."""
    from tests import helpers
    tenants = helpers.make_tenants(3)
    plan = helpers.plan_for(tenants, tile_cfg=4, split_k=4)
    sc.st_conv_run(plan)
    _sync(torch)
    fused = [t.dy.clone() for t in tenants]
    assert not torch.equal(fused[1], fused[3])        # same shape (batch 1), different weights and inputs
    for i, t in enumerate(tenants):
        t.clear()
        solo = helpers.plan_for([t], tile_cfg=4, split_k=4)
        sc.st_conv_run(solo)
        _sync(torch)
        assert torch.equal(t.dy, fused[i]), f"tenant {i}: solo != fused"


def test_split_k_is_deterministic(torch):
    """The split-K hand-off crosses XCDs (partial tiles written by one workgroup, summed by another).  More than a
    thousand launches, rotating through three copies of the tensors (so operands and workspaces are not simply cache
    resident from the launch before) and two plans with different split factors; every output is compared bit for
    bit with the first launch of its plan, stopping at the first mismatch."""
    from tests import helpers
    copies = [helpers.make_tenants(2) for _ in range(3)]
    plans = {split: [helpers.plan_for(c, split_k=split) for c in copies] for split in (6, 4)}
    first = {}
    for split, ps in plans.items():
        sc.st_conv_run(ps[0])
        _sync(torch)
        first[split] = [t.dy.clone() for t in copies[0]]
        for i, t in enumerate(copies[0]):
            helpers.check_tenant(t, f"split-K {split} tenant {i}")
    launches = 0
    for rnd in range(44):
        for split, ps in plans.items():
            # a burst of back-to-back launches on rotating copies, then one check per copy
            for c in copies:
                for t in c:
                    t.clear()
            for rep in range(4):
                for p in ps:
                    sc.st_conv_run(p)
                    launches += 1
            _sync(torch)
            for ci, c in enumerate(copies):
                for i, t in enumerate(c):
                    assert torch.equal(t.dy, first[split][i]), f"round {rnd} split {split} copy {ci} tenant {i}: output changed"
    assert launches >= 1000


@pytest.mark.parametrize("cfg", [1, 3, 4])
@pytest.mark.parametrize("target_items", [128, 256])
def test_configs_planned_for_a_share_of_the_gpu(torch, cfg, target_items):
    """The plans that the forms with several batches in flight use (the planner fills 128 or 256 workgroup slots
    instead of the whole chip): full-size configurations, every element against the oracle."""
    from tests import helpers
    tenants = helpers.make_tenants(cfg)
    plan = helpers.plan_for(tenants, target_items=target_items)
    sc.st_conv_run(plan)
    _sync(torch)
    worst = max(helpers.check_tenant(t, f"cfg{cfg} target_items={target_items} tenant {i}") for i, t in enumerate(tenants))
    print(f"cfg{cfg} target_items={target_items}: max |gpu-oracle| = {worst:.3e}")


def test_per_tenant_plan_baselines(torch):
    """Baselines with one plan per tenant (each planned alone) match the oracle too."""
    from tests import helpers
    tenants = helpers.make_tenants(2)
    plans = [helpers.plan_for([t]) for t in tenants]
    sc.st_conv_run_plans_time_only(plans)
    _sync(torch)
    for i, t in enumerate(tenants):
        helpers.check_tenant(t, f"time-only, own plan, tenant {i}")
        t.clear()
    streams = [torch.cuda.Stream() for _ in tenants]
    sc.st_conv_run_plans_space_only(plans, streams[:3])        # fewer streams than plans
    _sync(torch)
    for i, t in enumerate(tenants):
        helpers.check_tenant(t, f"space-only, own plan, tenant {i}")
    # free-running form, one call and the native loop over many rounds (the latter issues from several host threads)
    for rounds in (0, 1, 50):
        for t in tenants:
            t.clear()
        if rounds == 0:
            sc.st_conv_run_plans_on_streams(plans, streams)
        else:
            sc.st_conv_run_plans_on_streams_many(plans, streams, rounds)
        _sync(torch)
        for i, t in enumerate(tenants):
            helpers.check_tenant(t, f"free-running, {rounds} rounds, tenant {i}")
    sc.st_conv_run_plans_time_only([])
    sc.st_conv_run_plans_space_only([], streams)
    sc.st_conv_run_plans_on_streams_many([], streams, 3)


def test_split_k_workspace_is_not_stale_across_inputs(torch):
    """The split-K workspace is reused by every run of a plan.  Feeding different inputs through the same
    plan (rebind) must give the new inputs' result: a read of a stale cached partial would reproduce the
    previous run's values instead."""
    from tests import helpers
    shape = synth.config_shapes(2)[3]            # 49 x 512 x 4608: split-K territory
    a = helpers.Tenant(shape, synth.gen_input(93, 0, 0, shape), synth.gen_weight(93, 0, 0, shape))
    b = helpers.Tenant(shape, synth.gen_input(93, 1, 0, shape), synth.gen_weight(93, 1, 0, shape))
    plan = helpers.plan_for([a], tile_cfg=4, split_k=9)
    assert sc.st_conv_plan_tenant_info(plan, 0).split_k == 9
    for rep in range(3):
        sc.st_conv_plan_rebind(plan, 0, x=a.dx, w=a.dw, y=a.dy)
        sc.st_conv_run(plan)
        _sync(torch)
        helpers.check_tenant(a, f"rep {rep} inputs A")
        sc.st_conv_plan_rebind(plan, 0, x=b.dx, w=b.dw, y=b.dy)
        sc.st_conv_run(plan)
        _sync(torch)
        helpers.check_tenant(b, f"rep {rep} inputs B")
        assert not torch.equal(a.dy, b.dy)
        a.clear(); b.clear()


@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
def test_epilogue_residual_relu(torch, out_dtype):
    from tests import helpers
    shapes = [ConvShape(1, 64, 14, 14, 96, 1, 1, 1, 0, "bf16", out_dtype), ConvShape(2, 32, 9, 9, 48, 3, 3, 1, 1, "bf16", out_dtype)]
    tenants = []
    for t, s in enumerate(shapes):
        res = synth.to_storage(synth.uniform_pm1(synth.stream_state(91, t, 0, 3), s.N * s.K * s.P * s.Q), out_dtype)
        tenants.append(helpers.Tenant(s, synth.gen_input(91, t, 0, s), synth.gen_weight(91, t, 0, s, 2.0),
                                      residual=res.reshape(s.N, s.K, s.P, s.Q), relu=True))
    for opts in ({}, {"tile_cfg": 4, "split_k": 2}):
        for t in tenants:
            t.clear()
        plan = helpers.plan_for(tenants, **opts)
        sc.st_conv_run(plan)
        _sync(torch)
        for i, t in enumerate(tenants):
            helpers.check_tenant(t, f"epilogue tenant {i} {opts}")
            assert (t.result() >= 0).all()


def test_rebind_and_empty_plan(torch):
    from tests import helpers
    empty = sc.st_conv_plan([])
    sc.st_conv_run(empty)
    sc.st_conv_run_time_only(empty)
    sc.st_conv_run_space_only(empty, [torch.cuda.Stream()])
    assert sc.st_conv_plan_info(empty).n_items == 0
    a, b = helpers.make_tenants(1)
    plan = helpers.plan_for([a])
    sc.st_conv_run(plan)
    _sync(torch)
    helpers.check_tenant(a, "before rebind")
    sc.st_conv_plan_rebind(plan, 0, x=b.dx, w=b.dw, y=b.dy)
    sc.st_conv_run(plan)
    _sync(torch)
    helpers.check_tenant(b, "after rebind")


@pytest.mark.parametrize("C,dtype", [(24, "bf16"), (5, "bf16"), (16, "f16"), (12, "f32"), (3, "f32")])
def test_maxpool(torch, C, dtype):
    from oracle import oracle
    from tests import helpers
    x = synth.to_storage(synth.uniform_pm1(synth.stream_state(92, C, 0, 1), 2 * C * 15 * 14), dtype).reshape(2, C, 15, 14)
    dx = helpers.to_device_nhwc(x, dtype)
    dy = torch.zeros((2, 8, 7, C), dtype=helpers.torch_dtype(dtype), device="cuda")
    sc.st_maxpool_nhwc(dx, dy, 2, 15, 14, C, 3, 2, 1, dtype)
    _sync(torch)
    assert np.array_equal(helpers.from_device_nhwc(dy), oracle.maxpool2d(x, 3, 2, 1))


def test_plan_cache_dynamic_arrival(torch):
    """The ready set changes from step to step (Section 4: the scheduler merges whichever kernels are ready).
    Plans come from the cache; a hit is rebound to that step's buffers.  Every step's outputs are checked against
    the oracle; two steps with the same key and different buffers are queued back to back without a host
    synchronisation in between, and both must come out right (the rebind is ordered on the stream)."""
    from tests import helpers
    shapes = [ConvShape(1, 32, 14, 14, 48, 3, 3, 1, 1, "bf16", "f32"), ConvShape(2, 64, 7, 7, 64, 1, 1, 1, 0, "bf16", "f32"),
              ConvShape(1, 16, 20, 20, 40, 3, 3, 2, 1, "bf16", "bf16"), ConvShape(1, 128, 7, 7, 128, 3, 3, 1, 1, "bf16", "f32"),
              ConvShape(1, 24, 9, 9, 16, 5, 5, 1, 2, "f16", "f32")]
    # two variants (inputs and output buffers) per tenant, same weights
    var = [[helpers.Tenant(s, synth.gen_input(92, t, v, s), synth.gen_weight(92, t, 0, s)) for v in range(2)]
           for t, s in enumerate(shapes)]
    refs = [[v.reference() for v in tv] for tv in var]
    cache = sc.PlanCache(4)
    rng = np.random.default_rng(7)
    stream = torch.cuda.Stream()
    for step in range(14):
        ready = [t for t in range(len(shapes)) if rng.random() < 0.6] or [int(rng.integers(len(shapes)))]
        pick = [int(rng.integers(2)) for _ in ready]
        tenants = [var[t][v] for t, v in zip(ready, pick)]
        for tn in tenants:
            tn.clear()
        torch.cuda.synchronize()
        plan, hit = cache.get([tn.desc() for tn in tenants], stream)
        sc.st_conv_run(plan, stream)
        # the same ready set again at once, on the other variant's buffers, without waiting
        other = [var[t][1 - v] for t, v in zip(ready, pick)]
        for tn in other:
            tn.clear()
        plan2, hit2 = cache.get([tn.desc() for tn in other], stream)
        assert hit2 and plan2.handle == plan.handle
        sc.st_conv_run(plan2, stream)
        torch.cuda.synchronize()
        for t, v, a, b in zip(ready, pick, tenants, other):
            for tn, ref in ((a, refs[t][v]), (b, refs[t][1 - v])):
                got = tn.result()
                assert (np.abs(got - ref) <= helpers.tolerance(tn.shape, ref)).all(), f"step {step} tenant {t}"
    st = cache.stats()
    assert st.hits >= 14 and st.misses >= 2 and st.size <= 4
    cache.destroy()


def test_pipeline_keeps_independent_batches_in_flight(torch):
    """A ring of four streams, four sets of tensors, plans made for a quarter of the GPU each: twelve launches queued
    round-robin without waiting, one synchronisation, every batch's outputs checked against the oracle."""
    from tests import helpers
    pipe = sc.Pipeline(4)
    assert pipe.slots == 128 and sc.Pipeline(1).slots == 0 and sc.Pipeline(2).slots == 256
    batches = [helpers.make_tenants(2) for _ in range(4)]      # same seeded tensors, separate device buffers
    plans = [helpers.plan_for(b, target_items=pipe.slots) for b in batches]
    for rnd in range(3):
        for b in batches:
            for t in b:
                t.clear()
        torch.cuda.synchronize()
        seen = set()
        for i in range(4):
            stream = pipe.next()
            seen.add(stream)
            sc.st_conv_run(plans[i], stream)
        assert len(seen) == 4
        pipe.sync()
        if rnd == 1:          # the combined call: next stream + launch
            for i in range(4):
                pipe.run(plans[i])
            pipe.sync()
        if rnd == 2:          # the native loop: every plan twice over, then often enough for the issuing threads
            pipe.run_many(plans, 2)
            pipe.sync()
            pipe.run_many(plans, 40)
            pipe.sync()
        for bi, b in enumerate(batches):
            for ti, t in enumerate(b):
                helpers.check_tenant(t, f"round {rnd} batch {bi} tenant {ti}")
    with pytest.raises(sc.StError):
        sc.Pipeline(0)
    pipe.destroy()


def test_tensor_just_below_the_size_limit(torch):
    """The largest input the library accepts: x just below 2^31 bytes (1 x 4000 x 4000 x 64 bf16 = 2.048e9 bytes), so
    byte offsets use nearly the whole 32-bit range; y is 1.02e9 bytes of fp32.  Bands of output rows at the top, the
    middle and the bottom of the image (the last addresses) are compared element by element with the oracle run on
    the matching band of input rows (a 3x3 conv reads one row above and below)."""
    from oracle import oracle
    H = W = 4000
    C, K = 64, 16
    g = torch.Generator(device="cuda").manual_seed(190100041)
    x = (torch.rand((1, H, W, C), device="cuda", generator=g) * 2 - 1).to(torch.bfloat16)
    w = (torch.randn((K, 3, 3, C), device="cuda", generator=g) / (9 * C) ** 0.5).to(torch.bfloat16)
    y = torch.full((1, H, W, K), float("nan"), dtype=torch.float32, device="cuda")
    assert x.numel() * 2 < 2 ** 31 and x.numel() * 2 > 0.95 * 2 ** 31
    plan = sc.st_conv_plan([sc.make_desc(1, C, H, W, K, 3, 3, 1, 1, "bf16", "f32", x, w, y)], keep=[x, w, y])
    assert int(sc.st_conv_plan_info(plan).flops) == 2 * H * W * K * 9 * C
    sc.st_conv_run(plan)
    _sync(torch)
    assert bool(torch.isfinite(y).all()), "an output element was never written"
    w64 = w.double().cpu().numpy().transpose(0, 3, 1, 2)
    worst = 0.0
    for a, b in ((0, 6), (1997, 2003), (H - 6, H)):
        lo, hi = max(a - 1, 0), min(b + 1, H)
        band = x[:, lo:hi].double().cpu().numpy().transpose(0, 3, 1, 2)
        ref = oracle.conv2d(band, w64, 1, 1)[:, :, a - lo:b - lo, :]            # rows a..b-1 of the full result
        got = y[:, a:b].double().cpu().numpy().transpose(0, 3, 1, 2)
        err = np.abs(got - ref)
        assert (err <= 1e-4 * (np.abs(ref) + 1.0)).all(), f"rows {a}..{b}: max err {err.max():.3e}"
        worst = max(worst, float(err.max()))
    print(f"maximum-size tensor: worst error {worst:.3e}")
    # one element more per pixel row would cross the limit
    with pytest.raises(sc.StError):
        sc.st_conv_plan([sc.make_desc(1, C, H + 200, W, K, 3, 3, 1, 1, "bf16", "f32", x, w, y)], sc.plan_opts(host_only=1))


DEGENERATE = [
    ConvShape(1, 1, 1, 1, 1, 1, 1, 1, 0, "f32", "f32"),          # a single multiply
    ConvShape(1, 1, 1, 1, 1, 1, 1, 1, 0, "bf16", "bf16"),
    ConvShape(1, 8, 1, 1, 8, 1, 1, 1, 0, "bf16", "f32"),         # one pixel: a matrix-vector product
    ConvShape(2, 16, 3, 3, 5, 3, 3, 5, 0, "f16", "f32"),         # stride larger than the image: one output pixel
    ConvShape(1, 8, 2, 2, 3, 3, 3, 1, 3, "bf16", "f32"),         # padding wider than the image: most taps read zeros
    ConvShape(1, 2, 1, 40, 1, 1, 1, 1, 0, "f32", "f32"),         # one row, one filter
    ConvShape(1, 16, 5, 1, 4, 5, 1, 1, 2, "bf16", "f32"),        # one column, tall filter
    ConvShape(3, 1, 6, 6, 2, 2, 2, 2, 0, "f32", "f32"),          # one channel
]


def test_degenerate_shapes(torch):
    """Single pixels, single channels and filters, strides and paddings larger than the image: alone and fused."""
    from tests import helpers
    tenants = [helpers.Tenant(s, synth.gen_input(95, t, 0, s), synth.gen_weight(95, t, 0, s)) for t, s in enumerate(DEGENERATE)]
    for t in tenants:                                   # each alone
        sc.st_conv_run(helpers.plan_for([t]))
    _sync(torch)
    for i, t in enumerate(tenants):
        helpers.check_tenant(t, f"degenerate[{i}] alone {t.shape}")
        t.clear()
    plan = helpers.plan_for(tenants)                    # all in one launch
    sc.st_conv_run(plan)
    _sync(torch)
    for i, t in enumerate(tenants):
        helpers.check_tenant(t, f"degenerate[{i}] fused {t.shape}")


def test_many_tenants_in_one_launch(torch):
    """300 small tenants (more than 255, more than there are compute units), distinct weights each, in one fused launch."""
    from tests import helpers
    shapes = [ConvShape(1, 16, 6, 5 + (t % 3), 8 + 8 * (t % 2), 3, 3, 1, 1, "bf16", "f32") for t in range(300)]
    tenants = [helpers.Tenant(s, synth.gen_input(96, t, 0, s), synth.gen_weight(96, t, 0, s)) for t, s in enumerate(shapes)]
    plan = helpers.plan_for(tenants)
    assert int(sc.st_conv_plan_info(plan).n_tenants) == 300
    sc.st_conv_run(plan)
    _sync(torch)
    for i, t in enumerate(tenants):
        helpers.check_tenant(t, f"tenant {i} of 300")


def _random_shapes(seed: int, n: int):
    """Seeded assortment of small layers: every dtype, odd sizes, strides 1-3, paddings 0-3, filters 1x1 to 5x5 (square
    or not), channel counts that are and are not multiples of the 16-byte vector."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        dtype = ("bf16", "f16", "f32")[int(rng.integers(3))]
        out_dtype = "f32" if rng.random() < 0.6 else dtype
        R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        stride, pad = int(rng.integers(1, 4)), int(rng.integers(0, 4))
        H, W = int(rng.integers(1, 20)), int(rng.integers(1, 20))
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        C = int(rng.choice([1, 3, 4, 8, 12, 16, 24, 40, 64, 72]))
        K = int(rng.choice([1, 5, 8, 16, 24, 40, 64, 100, 136]))
        out.append(ConvShape(int(rng.integers(1, 4)), C, H, W, K, R, S, stride, pad, dtype, out_dtype))
    return out


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_shapes_in_one_launch(torch, seed):
    """Forty seeded random layers in one fused launch (planner's own choices), and again with a forced small tile and
    split-K: every element against the oracle."""
    from tests import helpers
    shapes = _random_shapes(seed, 40)
    tenants = [helpers.Tenant(s, synth.gen_input(99, t, seed, s), synth.gen_weight(99, t, seed, s), relu=bool(t % 3 == 0))
               for t, s in enumerate(shapes)]
    for opts in ({}, {"tile_cfg": 5, "split_k": 2}, {"tile_cfg": 1, "order": 2}):
        for t in tenants:
            t.clear()
        plan = helpers.plan_for(tenants, **opts)
        sc.st_conv_run(plan)
        _sync(torch)
        for i, t in enumerate(tenants):
            helpers.check_tenant(t, f"seed {seed} tenant {i} {t.shape} opts={opts}")
