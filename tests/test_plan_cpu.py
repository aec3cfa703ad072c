"""Host-side tests of the C ABI (no GPU, no compute calls): exports, validation, derived sizes and the
bit-exact work lists, checked against an independent re-derivation in Python."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_1901_00041_amd import st_conv as sc
from paper_1901_00041_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = dict(x=0x10000, w=0x20000, y=0x30000)


def _desc(s, **kw):
    args = dict(x=FAKE["x"], w=FAKE["w"], y=FAKE["y"], residual=None, epilogue=0)
    args.update(kw)
    return sc.make_desc(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, s.dtype, s.out_dtype,
                        args["x"], args["w"], args["y"], args["residual"], args["epilogue"])


def _host_plan(shapes, **opts):
    return sc.st_conv_plan([_desc(s) for s in shapes], sc.plan_opts(host_only=1, **opts))


def test_library_exports_every_declared_symbol():
    import glob
    headers = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    assert headers, "no public header"
    declared = set()
    for h in headers:
        declared |= set(re.findall(r"\b(st_[a-z0-9_]+)\s*\(", open(h).read()))
    assert not any("probe" in name for name in declared), "measurement probes do not belong in the public ABI"
    assert {"st_conv_plan", "st_conv_run", "st_conv_run_time_only", "st_conv_run_space_only"} <= declared
    lib = ctypes.CDLL(sc.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} is declared in include/ but not exported"
    assert declared == set(sc.EXPORTS), (declared ^ set(sc.EXPORTS))


def test_section41_worked_example_dims():
    # Section 4.1: 3x3, 128 -> 128 channels, 16x16 outputs  =>  M=256, N=128, K=1152
    p = _host_plan([synth.ConvShape(1, 128, 16, 16, 128, 3, 3, 1, 1)])
    ti = sc.st_conv_plan_tenant_info(p, 0)
    assert (ti.P, ti.Q, ti.M, ti.Ngemm, ti.Kgemm, ti.flops) == (16, 16, 256, 128, 1152, 75497472)
    # Table 1's other two shapes as 1x1 convolutions
    ti = sc.st_conv_plan_tenant_info(_host_plan([synth.ConvShape(1, 256, 16, 16, 256, 1, 1, 1, 0)]), 0)
    assert (ti.M, ti.Ngemm, ti.Kgemm) == (256, 256, 256)
    ti = sc.st_conv_plan_tenant_info(_host_plan([synth.ConvShape(1, 512, 1, 1, 512, 1, 1, 1, 0)]), 0)
    assert (ti.M, ti.Ngemm, ti.Kgemm) == (1, 512, 512)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_config_totals_match_generator(cfg):
    shapes = synth.config_shapes(cfg)
    p = _host_plan(shapes)
    info = sc.st_conv_plan_info(p)
    assert info.n_tenants == len(shapes) and info.host_only == 1
    assert info.flops == sum(s.flops for s in shapes) and info.bytes == sum(s.bytes for s in shapes)
    for t, s in enumerate(shapes):
        ti = sc.st_conv_plan_tenant_info(p, t)
        assert (ti.M, ti.Ngemm, ti.Kgemm) == s.gemm and (ti.P, ti.Q) == (s.P, s.Q)


def _xcd_blocks(shape, ti):
    """The block grid restated: most blocks first (at most 8, powers of two per side, no more blocks than tiles per
    side), then fewest bytes fetched over all XCDs (activations once per filter-block column, filters once per
    pixel-block row), then the smaller pixel-block count."""
    es = 4 if shape.dtype == "f32" else 2
    w_bytes = ti.Ngemm * ti.Kgemm * es
    x_bytes = shape.N * shape.C * shape.H * shape.W * es
    cands = [(a, b) for a in (1, 2, 4, 8) for b in (1, 2, 4, 8) if a * b <= 8 and a <= ti.tiles_m and b <= ti.tiles_n]
    return min(cands, key=lambda ab: (-ab[0] * ab[1], ab[1] * x_bytes + ab[0] * w_bytes, ab[0]))


def _xcd_deal(rows, phase, ti):
    """The placement rule restated: rows (tenant, k, tile_m, tile_n, 0) in nested order are dealt to launch
    positions; position q (XCD (phase+q) % 8) takes the next row whose block prefers that XCD, else the next
    row of the XCD with most rows left (lowest XCD on ties)."""
    a, b = ti.xcd_blocks_m, ti.xcd_blocks_n
    if a * b <= 1 or len(rows) < 2:
        return list(rows)
    buckets = [[] for _ in range(8)]
    for r in rows:
        g = (r[2] * a // ti.tiles_m) * b + (r[3] * b // ti.tiles_n)
        buckets[g % 8].append(r)
    out = []
    for q in range(len(rows)):
        x = (phase + q) % 8
        if not buckets[x]:
            x = max(range(8), key=lambda c: (len(buckets[c]), -c))
        out.append(buckets[x].pop(0))
    return out


def _expected_tenant_major(plan, n_tenants, shapes=None):
    """Independent enumeration from the per-tenant summary only: per tenant the nested order pixel tile,
    filter tile, K slice, dealt to XCDs with each tenant's own launch starting at its first item."""
    rows = []
    for t in range(n_tenants):
        ti = sc.st_conv_plan_tenant_info(plan, t)
        mt, nt, kb = sc.st_tile_shape(ti.tile_cfg)
        assert (mt, nt) == (ti.MT, ti.NT)
        if ti.row_tiled:       # pixel tiles are segments of single output rows
            assert ti.rows_per_tile >= 1 and ti.split_k == 1
            assert ti.tiles_m == (ti.M // (ti.P * ti.Q)) * -(-ti.P // ti.rows_per_tile) * -(-ti.Q // mt)
        else:
            assert ti.tiles_m == -(-ti.M // mt)
        assert ti.tiles_n == -(-ti.Ngemm // nt)
        assert ti.k_steps_per_split == -(-ti.k_steps // ti.split_k)
        assert (ti.split_k - 1) * ti.k_steps_per_split < ti.k_steps, "an empty K slice"
        assert ti.item_begin == len(rows) and ti.item_count == ti.tiles_m * ti.tiles_n * ti.split_k
        mine = [(t, s, tm, tn, 0) for tm in range(ti.tiles_m) for tn in range(ti.tiles_n) for s in range(ti.split_k)]
        if shapes is not None:
            assert (ti.xcd_blocks_m, ti.xcd_blocks_n) == _xcd_blocks(shapes[t], ti)
        rows.extend(_xcd_deal(mine, 0, ti))
    return np.array(rows, dtype=np.int64).reshape(-1, 5)


def _as_rows(items):
    return np.stack([items[f].astype(np.int64) for f in ("tenant", "k_split_idx", "tile_m", "tile_n", "reserved")], axis=1)


@pytest.mark.parametrize("cfg,opts", [(1, {}), (2, {}), (3, {}), (4, {}), (2, {"tile_cfg": 6, "split_k": 5}),
                                      (4, {"tile_cfg": 1}), (3, {"order": 1}), (4, {"split_k": 3, "target_items": 64}),
                                      (4, {"order": 2}), (2, {"order": 2})])
def test_work_lists_bit_exact(cfg, opts):
    shapes = synth.config_shapes(cfg)
    p = _host_plan(shapes, **opts)
    want = _expected_tenant_major(p, len(shapes), shapes)
    tenant_major = _as_rows(sc.st_conv_plan_worklist(p, 1))
    assert np.array_equal(tenant_major, want)
    fused = _as_rows(sc.st_conv_plan_worklist(p, 0))
    assert sc.st_conv_plan_info(p).n_items == len(want) == len(fused)
    # every (tenant, tile, slice) exactly once: the fused list is a permutation of the tenant-major one
    assert np.array_equal(np.unique(fused, axis=0), np.unique(want, axis=0)) and len(np.unique(fused, axis=0)) == len(want)
    if opts.get("order") == 1:
        assert np.array_equal(fused, want)
    if opts.get("order") == 2:
        # equal progress: the tenant furthest behind its share goes next ((emitted + 1) / count smallest, lowest
        # tenant on ties), taking its items in tenant-major order -- restated here with exact fractions
        from fractions import Fraction
        counts = [int(sc.st_conv_plan_tenant_info(p, t).item_count) for t in range(len(shapes))]
        begins = [int(sc.st_conv_plan_tenant_info(p, t).item_begin) for t in range(len(shapes))]
        emitted = [0] * len(shapes)
        for q in range(len(want)):
            t = min((t for t in range(len(shapes)) if emitted[t] < counts[t]),
                    key=lambda t: (Fraction(emitted[t] + 1, counts[t]), t))
            assert np.array_equal(fused[q], want[begins[t] + emitted[t]]), f"position {q}"
            emitted[t] += 1
    # K coverage: the slices of a tile tile [0, k_steps) without gap or overlap, and cover Kgemm
    for t, s in enumerate(shapes):
        ti = sc.st_conv_plan_tenant_info(p, t)
        kb = sc.st_tile_shape(ti.tile_cfg)[2]
        es = 4 if s.dtype == "f32" else 2
        if ti.row_tiled:
            assert ti.k_steps == s.R      # one filter row per step
            continue
        assert ti.k_steps == -(-ti.Kgemm * es // kb)
        covered = 0
        for i in range(ti.split_k):
            b = i * ti.k_steps_per_split
            e = min(ti.k_steps, b + ti.k_steps_per_split)
            assert b == covered and e > b
            covered = e
        assert covered == ti.k_steps and covered * kb >= ti.Kgemm * es
    # determinism: the same descriptors give the same lists
    p2 = _host_plan(shapes, **opts)
    assert np.array_equal(_as_rows(sc.st_conv_plan_worklist(p2, 0)), fused)


def test_fused_list_keeps_tile_blocks_on_one_xcd():
    """Workgroup b of a launch runs on XCD b mod 8.  For every tenant whose items form one run of the fused list and
    whose 8 blocks hold equally many items, every block sits on exactly one XCD; for every other tenant with 8 blocks,
    most of each block's items sit on the block's own XCD (the rest were dealt to XCDs that had run dry)."""
    exact = loose = 0
    for cfg in (2, 3, 4):
        shapes = synth.config_shapes(cfg)
        p = _host_plan(shapes)
        fused = _as_rows(sc.st_conv_plan_worklist(p, 0))
        for t in range(len(shapes)):
            ti = sc.st_conv_plan_tenant_info(p, t)
            pos = np.nonzero(fused[:, 0] == t)[0]
            a, b = ti.xcd_blocks_m, ti.xcd_blocks_n
            if a * b != 8 or len(pos) != pos[-1] - pos[0] + 1:
                continue
            block = (fused[pos, 2] * a // ti.tiles_m) * b + (fused[pos, 3] * b // ti.tiles_n)
            sizes = [int((block == g).sum()) for g in range(8)]
            for g in range(8):
                on = pos[block == g] % 8
                if len(set(sizes)) == 1:
                    assert len(set(on.tolist())) == 1, f"cfg {cfg} tenant {t} block {g} spans several XCDs"
                else:
                    assert (on == g).sum() * 2 >= len(on) or sizes[g] > 2 * min(sizes), f"cfg {cfg} tenant {t} block {g}"
            exact += len(set(sizes)) == 1
            loose += len(set(sizes)) != 1
    assert exact > 0 and exact + loose > 3


def test_fused_order_longest_first():
    shapes = synth.config_shapes(4)
    p = _host_plan(shapes)
    items = sc.st_conv_plan_worklist(p, 0)
    steps = []
    for it in items:
        ti = sc.st_conv_plan_tenant_info(p, int(it["tenant"]))
        b = int(it["k_split_idx"]) * ti.k_steps_per_split
        steps.append((min(ti.k_steps, b + ti.k_steps_per_split) - b, ti.tile_cfg))
    # within one tile shape, items with more K steps never come later than items with fewer
    for cfg in set(c for _, c in steps):
        seq = [s for s, c in steps if c == cfg]
        assert seq == sorted(seq, reverse=True)


def test_row_tile_is_chosen_for_the_stem_only_when_eligible():
    stem = synth.ConvShape(1, 3, 224, 224, 64, 7, 7, 2, 3)
    p = _host_plan([stem, synth.ConvShape(1, 3, 30, 26, 64, 7, 7, 2, 3), synth.ConvShape(1, 64, 56, 56, 64, 3, 3, 1, 1)])
    a, b, c = (sc.st_conv_plan_tenant_info(p, t) for t in range(3))
    assert a.row_tiled == 1 and (a.MT, a.NT) == (128, 64) and a.tiles_m == 112 // a.rows_per_tile and a.k_steps == 7
    assert b.row_tiled == 0      # image rows are not a multiple of 16 bytes: element-wise gather kernel
    assert c.row_tiled == 0


def test_tile_family_is_sane():
    n = sc.st_tile_count()
    assert n >= 4
    for i in range(n):
        mt, nt, kb = sc.st_tile_shape(i)
        assert mt % 16 == 0 and nt % 16 == 0 and kb in (64, 128, 256)
    with pytest.raises(sc.StError):
        sc.st_tile_shape(n)


def test_validation_errors():
    good = synth.ConvShape(1, 16, 8, 8, 16, 3, 3, 1, 1)

    def status(desc, opts=None):
        try:
            sc.st_conv_plan([desc], opts or sc.plan_opts(host_only=1))
        except sc.StError as e:
            assert str(e)            # message is populated
            return e.status
        return sc.ST_OK

    import dataclasses
    assert status(_desc(good)) == sc.ST_OK
    for field, val in (("N", 0), ("C", -1), ("H", 0), ("K", 0), ("R", 0), ("stride", 0), ("pad", -1)):
        assert status(_desc(dataclasses.replace(good, **{field: val}))) == sc.ST_ERR_INVALID_ARG, field
    assert status(_desc(dataclasses.replace(good, R=11))) == sc.ST_ERR_INVALID_ARG          # empty output
    assert status(_desc(good, x=None)) == sc.ST_ERR_INVALID_ARG
    assert status(_desc(good, y=FAKE["x"])) == sc.ST_ERR_INVALID_ARG                        # y aliases x
    assert status(_desc(good, epilogue=sc.ST_EPI_RESIDUAL)) == sc.ST_ERR_INVALID_ARG       # no residual pointer
    assert status(_desc(good, epilogue=8)) == sc.ST_ERR_UNSUPPORTED
    d = _desc(good); d.in_dtype = 7
    assert status(d) == sc.ST_ERR_UNSUPPORTED
    d = _desc(good); d.out_dtype = sc.ST_DT_F16            # neither f32 nor in_dtype (bf16)
    assert status(d) == sc.ST_ERR_UNSUPPORTED
    d = _desc(good); d.layout = 3
    assert status(d) == sc.ST_ERR_UNSUPPORTED
    d = _desc(good); d.layout = sc.ST_LAYOUT_NCHW_KCRS     # named in the header, not implemented
    assert status(d) == sc.ST_ERR_UNSUPPORTED
    d = _desc(good); d.reserved = 1
    assert status(d) == sc.ST_ERR_INVALID_ARG
    assert status(_desc(synth.ConvShape(64, 1024, 256, 256, 8, 1, 1, 1, 0))) == sc.ST_ERR_UNSUPPORTED   # 2^32 elements
    assert status(_desc(good), sc.plan_opts(host_only=1, tile_cfg=99)) == sc.ST_ERR_INVALID_ARG
    # NULL plan output and negative tenant count
    assert sc.lib().st_conv_plan(None, 0, None, None) == sc.ST_ERR_INVALID_ARG
    out = ctypes.c_void_p()
    assert sc.lib().st_conv_plan(None, -1, None, ctypes.byref(out)) == sc.ST_ERR_INVALID_ARG and not out.value
    assert sc.lib().st_conv_plan(None, 2, None, ctypes.byref(out)) == sc.ST_ERR_INVALID_ARG and not out.value


def test_host_only_plan_refuses_to_run_and_empty_plan_is_ok():
    p = _host_plan(synth.config_shapes(1))
    with pytest.raises(sc.StError) as e:
        sc.st_conv_run(p)
    assert e.value.status == sc.ST_ERR_UNSUPPORTED
    for fn in (sc.st_conv_run_time_only,):
        with pytest.raises(sc.StError):
            fn(p)
    empty = sc.st_conv_plan([], sc.plan_opts(host_only=1))
    info = sc.st_conv_plan_info(empty)
    assert info.n_tenants == 0 and info.n_items == 0 and len(sc.st_conv_plan_worklist(empty, 0)) == 0
    with pytest.raises(sc.StError):
        sc.st_conv_plan_tenant_info(empty, 0)


def test_rebind_checks_on_host_plan():
    p = _host_plan(synth.config_shapes(1))
    sc.st_conv_plan_rebind(p, 1, x=0x50000)
    with pytest.raises(sc.StError):
        sc.st_conv_plan_rebind(p, 2, x=0x50000)            # tenant out of range
    with pytest.raises(sc.StError):
        sc.st_conv_plan_rebind(p, 0, y=FAKE["x"])          # would alias


def test_split_k_plan_on_two_streams_is_rejected():
    """A plan that owns a split-K workspace must not be in flight on two streams: the multi-stream calls refuse it
    before touching the device (host-only plans, made-up stream handles)."""
    deep = synth.config_shapes(2)[3]                       # 49 x 512 x 4608: split-K
    a = sc.st_conv_plan([_desc(deep)], sc.plan_opts(host_only=1, tile_cfg=5, split_k=4))
    b = sc.st_conv_plan([_desc(synth.config_shapes(1)[0])], sc.plan_opts(host_only=1, split_k=1))
    assert sc.st_conv_plan_info(a).workspace_bytes > 0 and sc.st_conv_plan_info(b).workspace_bytes == 0
    streams = [0x1000, 0x2000]
    for call in (lambda: sc.st_conv_run_plans_on_streams([a, a], streams),
                 lambda: sc.st_conv_run_plans_on_streams_many([b, a, a], streams, 3)):
        with pytest.raises(sc.StError) as e:
            call()
        assert e.value.status == sc.ST_ERR_INVALID_ARG and "workspace" in str(e.value)
    # the same plan twice on ONE stream is ordered by the stream: accepted as far as this check goes (the host-only
    # plan is then refused by the run itself)
    with pytest.raises(sc.StError) as e:
        sc.st_conv_run_plans_on_streams([a, b, a], [0x1000, 0x2000])      # a -> stream 0 both times
    assert e.value.status == sc.ST_ERR_UNSUPPORTED


def test_status_strings():
    assert sc.lib().st_status_string(0) == b"ST_OK" and sc.lib().st_status_string(2) == b"ST_ERR_UNSUPPORTED"


def test_plan_cache_hits_misses_eviction_and_rebinding():
    """Host-only plan cache: the key is everything but the pointers, in tenant order; a hit rebinds the cached
    plan to the new pointers; the least recently used plan goes first."""
    shapes = synth.config_shapes(2)
    cache = sc.PlanCache(2, sc.plan_opts(host_only=1))
    a = [_desc(s) for s in shapes]
    p1, hit = cache.get(a)
    assert not hit and sc.st_conv_plan_info(p1).n_tenants == 4
    # same shapes, other pointers: the same plan comes back, with the same work list
    items1 = _as_rows(sc.st_conv_plan_worklist(p1, 0)).copy()
    b = [_desc(s, x=0x50000 + 0x1000 * t, w=0x60000 + 0x1000 * t, y=0x70000 + 0x1000 * t) for t, s in enumerate(shapes)]
    p2, hit = cache.get(b)
    assert hit and p2.handle == p1.handle
    assert np.array_equal(_as_rows(sc.st_conv_plan_worklist(p2, 0)), items1)
    # a different ready set (subset, and another order) is a different key
    p3, hit = cache.get(a[:3])
    assert not hit and p3.handle != p1.handle
    st = cache.stats()
    assert (st.hits, st.misses, st.evictions, st.size, st.capacity) == (1, 2, 0, 2, 2)
    p4, hit = cache.get(a[::-1])                 # cache full: evicts the 4-tenant plan (least recently used)
    assert not hit
    st = cache.stats()
    assert (st.misses, st.evictions, st.size) == (3, 1, 2)
    _, hit = cache.get(a[:3])
    assert hit                                  # still cached
    _, hit = cache.get(a)
    assert not hit                              # was evicted, rebuilt
    # an epilogue bit or a residual pointer changes the key
    _, hit = cache.get([_desc(shapes[0])])
    assert not hit
    _, hit = cache.get([_desc(shapes[0], epilogue=sc.ST_EPI_RELU)])
    assert not hit
    # errors pass through and cache nothing
    before = cache.stats().misses
    with pytest.raises(sc.StError):
        cache.get([_desc(shapes[0], y=FAKE["x"])])          # y aliases x
    assert cache.stats().misses == before
    with pytest.raises(sc.StError):
        sc.PlanCache(0)
    cache.destroy()


def test_rebind_all_validates_and_keeps_shapes():
    shapes = synth.config_shapes(3)
    p = _host_plan(shapes)
    with pytest.raises(sc.StError):
        sc.st_conv_plan_rebind_all(p, [_desc(s) for s in shapes[:-1]])          # wrong tenant count
    with pytest.raises(sc.StError):
        sc.st_conv_plan_rebind_all(p, [_desc(s, y=FAKE["w"]) for s in shapes])  # y aliases w
    with pytest.raises(sc.StError):
        sc.st_conv_plan_rebind_all(p, [_desc(s, x=None) for s in shapes])       # NULL x
    sc.st_conv_plan_rebind_all(p, [_desc(s, x=0x90000) for s in shapes])
    assert sc.st_conv_plan_info(p).n_tenants == len(shapes)


def test_planner_bisection_matches_exhaustive_search():
    """The planner bisects over the candidate bounds; with ST_PLAN_EXHAUSTIVE=1 it evaluates every bound.  Both
    must choose the same tile, split and rows per tile for every tenant, on the five configurations and on
    random mixes of their layers."""
    rng = np.random.default_rng(5)
    pool = [s for cfg in (1, 2, 3, 4) for s in synth.config_shapes(cfg)] + [st.shape for st in synth.resnet50_steps()]
    cases = [synth.config_shapes(cfg) for cfg in (1, 2, 3, 4)]
    cases += [[pool[i] for i in rng.integers(len(pool), size=int(rng.integers(1, 20)))] for _ in range(40)]

    def summary(p, n):
        out = []
        for t in range(n):
            ti = sc.st_conv_plan_tenant_info(p, t)
            out.append((ti.tile_cfg, ti.split_k, ti.rows_per_tile, ti.item_count))
        return out

    for shapes in cases:
        for slots in (0, 64):
            os.environ.pop("ST_PLAN_EXHAUSTIVE", None)
            fast = summary(_host_plan(shapes, target_items=slots), len(shapes))
            os.environ["ST_PLAN_EXHAUSTIVE"] = "1"
            try:
                slow = summary(_host_plan(shapes, target_items=slots), len(shapes))
            finally:
                os.environ.pop("ST_PLAN_EXHAUSTIVE", None)
            assert fast == slow


def test_pipeline_share_table_and_argument_checks():
    """The planner share that goes with a pipeline depth is a pure table; creating a ring needs a device, so without
    one the call must fail with a status (never crash), and bad depths are rejected before any device call."""
    assert [sc.lib().st_pipeline_slots(d) for d in (0, 1, 2, 3, 4, 8)] == [0, 0, 256, 128, 128, 128]
    out = ctypes.c_void_p()
    assert sc.lib().st_pipeline_create(0, ctypes.byref(out)) == sc.ST_ERR_INVALID_ARG and not out.value
    assert sc.lib().st_pipeline_create(65, ctypes.byref(out)) == sc.ST_ERR_INVALID_ARG and not out.value
    assert sc.lib().st_pipeline_create(2, None) == sc.ST_ERR_INVALID_ARG
    st = sc.lib().st_pipeline_create(2, ctypes.byref(out))
    if st == sc.ST_OK:
        sc.lib().st_pipeline_destroy(out)
    else:
        assert st == sc.ST_ERR_DEVICE and not out.value and sc.lib().st_last_error_message()
    assert sc.lib().st_pipeline_sync(None) == sc.ST_ERR_INVALID_ARG
    assert sc.lib().st_pipeline_run(None, None) == sc.ST_ERR_INVALID_ARG


def test_default_plan_prefers_one_workgroup_per_compute_unit_when_the_model_says_so():
    """With the default slot target the planner also plans for 256 slots (one workgroup per compute unit, each 1.3x faster
    than beside a second one) and takes that plan when its modelled launch is shorter: config 3 (8 tenants of 3x3
    256->256 @14x14) becomes 224 tiles of 64x64 instead of 416 of 32x64; an explicit target keeps the caller's choice;
    config 4 (more than a thousand tiles either way) is unaffected."""
    shapes = synth.config_shapes(3)
    auto = sc.st_conv_plan([_desc(s) for s in shapes], sc.plan_opts(host_only=1))
    forced = sc.st_conv_plan([_desc(s) for s in shapes], sc.plan_opts(host_only=1, target_items=400))
    ia, ifo = sc.st_conv_plan_info(auto), sc.st_conv_plan_info(forced)
    assert ia.n_items <= 256 < ifo.n_items
    assert {(sc.st_conv_plan_tenant_info(auto, t).MT, sc.st_conv_plan_tenant_info(auto, t).NT) for t in range(len(shapes))} == {(64, 64)}
    assert {(sc.st_conv_plan_tenant_info(forced, t).MT, sc.st_conv_plan_tenant_info(forced, t).NT) for t in range(len(shapes))} == {(32, 64)}
    shapes4 = synth.config_shapes(4)
    a4 = sc.st_conv_plan_info(sc.st_conv_plan([_desc(s) for s in shapes4], sc.plan_opts(host_only=1)))
    f4 = sc.st_conv_plan_info(sc.st_conv_plan([_desc(s) for s in shapes4], sc.plan_opts(host_only=1, target_items=400)))
    assert a4.n_items == f4.n_items > 256
