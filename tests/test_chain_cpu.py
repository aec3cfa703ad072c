"""Host-side tests of the chain planner (no GPU, no compute calls): the queue holds every work item of every op exactly
once, stage-major; every op's threshold equals the number of work items its sequence has in earlier stages; every
queue entry depends only on entries before it; tiles are the ones st_conv_plan picks for the stage's ops alone."""
import numpy as np
import pytest

from paper_1901_00041_amd import st_conv as sc
from paper_1901_00041_amd import synth
from paper_1901_00041_amd.synth import ConvShape

FAKE = 0x10000


def _conv_desc(s, tag):
    base = FAKE * (4 * tag + 1)
    return sc.make_desc(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, s.dtype, s.out_dtype, base, base + FAKE, base + 2 * FAKE)


def _pool_desc(N, C, H, W, tag, dtype="bf16"):
    base = FAKE * (4 * tag + 1)
    return sc.make_desc(N, C, H, W, C, 3, 3, 2, 1, dtype, dtype, base, None, base + 2 * FAKE)


def _resnet_ops(n_tenants):
    """The benchmark's chain: every tenant's 53 layers plus the max-pool, stages as the stack module assigns them."""
    steps = synth.resnet50_steps()
    ops, tag = [], 0
    stage = -2
    prev_src = None
    for st in steps:
        # a projection conv and the conv1 that follows it read the same tensor: one stage
        stage = stage if (prev_src == st.src and not st.pool_after and ".conv1" in st.name) else stage + 2
        prev_src = st.src if ".proj" in st.name else None
        for t in range(n_tenants):
            tag += 1
            ops.append(sc.make_chain_op(sc.ST_OP_CONV, t, stage, _conv_desc(st.shape, tag)))
            if st.pool_after:
                tag += 1
                ops.append(sc.make_chain_op(sc.ST_OP_MAXPOOL, t, stage + 1, _pool_desc(st.shape.N, st.shape.K, st.shape.P, st.shape.Q, tag)))
    return ops


def _check_chain(ops, chain):
    info = chain.info()
    items = chain.worklist()
    assert info.n_ops == len(ops) and info.n_items == len(items)
    per_op = [chain.op_info(i) for i in range(len(ops))]
    # every op's items exactly once
    for i, oi in enumerate(per_op):
        mine = items[items["tenant"] == i]
        assert len(mine) == oi.item_count, i
        assert (oi.sequence, oi.stage, oi.kind) == (ops[i].sequence, ops[i].stage, ops[i].kind)
        if oi.kind == sc.ST_OP_CONV:
            ti = oi.tile
            want = {(s, m, n) for m in range(ti.tiles_m) for n in range(ti.tiles_n) for s in range(ti.split_k)}
            got = set(zip(mine["k_split_idx"].tolist(), mine["tile_m"].tolist(), mine["tile_n"].tolist()))
            assert got == want and len(mine) == len(want), i
        else:
            assert sorted(mine["tile_m"].tolist()) == list(range(oi.item_count)) and (mine["tile_n"] == 0).all()
    # an XCD's entries (or the one queue's) hold whole sequences (sequence s on XCD s mod n_queues).  One queue: stage
    # order.  Per XCD: 32 exclusive + 32 shared columns, each in stage order; a stage's entries are dealt to the columns
    # in turn, exclusive ones first, so its k-th entry sits in column k mod 64 and a stage of at most 32 entries never
    # touches a shared column
    qb = list(info.queue_begin)[:info.n_queues + 1]
    sb = list(info.shared_begin)[:info.n_queues]
    cols = chain.columns()
    assert qb[0] == 0 and qb[-1] == len(items) and info.n_queues in (1, 8)
    stage_of = np.array([ops[t].stage for t in items["tenant"]])
    if info.n_queues == 1:
        assert info.columns == 0 and len(cols) == 0 and sb[0] == qb[1]
        assert (np.diff(stage_of) >= 0).all()
    else:
        nc = info.columns
        assert nc == 32 and len(cols) == 8 * 2 * nc + 1 and cols[0] == 0 and cols[-1] == len(items) and (np.diff(cols.astype(np.int64)) >= 0).all()
        for q in range(8):
            assert qb[q] == cols[q * 2 * nc] and sb[q] == cols[q * 2 * nc + nc]
            assert all(ops[t].sequence % 8 == q for t in items["tenant"][qb[q]:qb[q + 1]])
            per_stage = {}
            for j in range(2 * nc):
                lo, hi = int(cols[q * 2 * nc + j]), int(cols[q * 2 * nc + j + 1])
                assert (np.diff(stage_of[lo:hi]) >= 0).all()
                for st in stage_of[lo:hi]:
                    per_stage.setdefault(int(st), [0] * (2 * nc))[j] += 1
            for st, cnt in per_stage.items():
                n = sum(cnt)
                assert cnt == [n // (2 * nc) + (1 if j < n % (2 * nc) else 0) for j in range(2 * nc)], (q, st, cnt)
    # thresholds: items of the op's sequence in strictly earlier stages
    for i, oi in enumerate(per_op):
        need = sum(p.item_count for j, p in enumerate(per_op) if p.sequence == oi.sequence and p.stage < oi.stage)
        assert oi.need == need, (i, oi.need, need)
    # progress: an entry waits only for entries of strictly earlier stages (the thresholds above); the one queue is
    # claimed in stage order and every column is worked through in stage order, so an unfinished entry of the lowest
    # unfinished stage is never behind an entry that waits
    return per_op


def test_resnet_chain_queue_and_thresholds():
    ops = _resnet_ops(3)
    chain = sc.Chain(ops, sc.plan_opts(host_only=1))
    info = chain.info()
    assert info.n_sequences == 3 and info.host_only == 1 and info.n_stages == 50      # 49 layer groups + the max-pool
    assert info.flops == 3 * 8174272512
    per_op = _check_chain(ops, chain)
    # a stage's tiles are what st_conv_plan picks for that stage's convolutions on their own
    by_stage = {}
    for i, op in enumerate(ops):
        if op.kind == sc.ST_OP_CONV:
            by_stage.setdefault(op.stage, []).append(i)
    for stage in (0, 2, 20, max(by_stage)):
        idx = by_stage[stage]
        plan = sc.st_conv_plan([ops[i].conv for i in idx], sc.plan_opts(host_only=1))
        for j, i in enumerate(idx):
            a, b = sc.st_conv_plan_tenant_info(plan, j), per_op[i].tile
            assert (a.tile_cfg, a.split_k, a.tiles_m, a.tiles_n, a.k_steps_per_split) == (b.tile_cfg, b.split_k, b.tiles_m, b.tiles_n, b.k_steps_per_split)
    with pytest.raises(sc.StError) as e:
        chain.run()
    assert e.value.status == sc.ST_ERR_UNSUPPORTED
    assert chain.aborted() is False
    chain.set_workgroups(info.workgroups)
    chain.set_workgroups(0)
    for bad in (-1, info.workgroups + 1):
        with pytest.raises(sc.StError) as e:
            chain.set_workgroups(bad)
        assert e.value.status == sc.ST_ERR_INVALID_ARG


@pytest.mark.parametrize("chain_queues,want", [(0, 8), (1, 1), (2, 8)])
def test_resnet_chain_one_queue_per_xcd(chain_queues, want):
    """Eight tenants: by default every XCD gets a queue of its own with one tenant's whole network in it."""
    ops = _resnet_ops(8)
    chain = sc.Chain(ops, sc.plan_opts(host_only=1, chain_queues=chain_queues))
    info = chain.info()
    assert info.n_queues == want and info.n_sequences == 8
    _check_chain(ops, chain)
    if want == 8:
        sizes = np.diff(np.array(list(info.queue_begin)))
        assert (sizes == sizes[0]).all() and sizes[0] * 8 == info.n_items      # equal tenants, equal queues


def test_chain_with_uneven_sequences_and_shared_stages():
    a = ConvShape(1, 64, 14, 14, 64, 3, 3, 1, 1, "bf16", "bf16")
    b = ConvShape(2, 32, 9, 9, 48, 1, 1, 1, 0, "bf16", "bf16")
    ops = [sc.make_chain_op(sc.ST_OP_CONV, 0, 0, _conv_desc(a, 1)),
           sc.make_chain_op(sc.ST_OP_CONV, 0, 5, _conv_desc(a, 2)),
           sc.make_chain_op(sc.ST_OP_CONV, 0, 5, _conv_desc(b, 3)),          # same stage, same sequence: independent
           sc.make_chain_op(sc.ST_OP_CONV, 2, 5, _conv_desc(b, 4)),          # sequence 1 has no ops at all
           sc.make_chain_op(sc.ST_OP_MAXPOOL, 2, 7, _pool_desc(2, 48, 9, 9, 5)),
           sc.make_chain_op(sc.ST_OP_CONV, 0, 9, _conv_desc(b, 6))]
    chain = sc.Chain(ops, sc.plan_opts(host_only=1))
    info = chain.info()
    assert (info.n_sequences, info.n_stages) == (3, 4)
    per_op = _check_chain(ops, chain)
    assert per_op[0].need == 0 and per_op[3].need == 0
    assert per_op[1].need == per_op[2].need == per_op[0].item_count
    assert per_op[4].need == per_op[3].item_count and per_op[4].item_count == -(-2 * 5 * 5 * (48 // 8) // 256)
    assert per_op[5].need == per_op[0].item_count + per_op[1].item_count + per_op[2].item_count
    empty = sc.Chain([], sc.plan_opts(host_only=1))
    assert empty.info().n_items == 0


def test_chain_validation():
    good = ConvShape(1, 16, 8, 8, 16, 3, 3, 1, 1, "bf16", "bf16")

    def status(op):
        try:
            sc.Chain([op], sc.plan_opts(host_only=1))
        except sc.StError as e:
            assert str(e)
            return e.status
        return sc.ST_OK

    assert status(sc.make_chain_op(sc.ST_OP_CONV, 0, 0, _conv_desc(good, 1))) == sc.ST_OK
    assert status(sc.make_chain_op(5, 0, 0, _conv_desc(good, 1))) == sc.ST_ERR_INVALID_ARG
    assert status(sc.make_chain_op(sc.ST_OP_CONV, -1, 0, _conv_desc(good, 1))) == sc.ST_ERR_INVALID_ARG
    assert status(sc.make_chain_op(sc.ST_OP_CONV, 4096, 0, _conv_desc(good, 1))) == sc.ST_ERR_INVALID_ARG
    assert status(sc.make_chain_op(sc.ST_OP_CONV, 0, -2, _conv_desc(good, 1))) == sc.ST_ERR_INVALID_ARG
    bad = _conv_desc(good, 1)
    bad.N = 0
    assert status(sc.make_chain_op(sc.ST_OP_CONV, 0, 0, bad)) == sc.ST_ERR_INVALID_ARG
    assert status(sc.make_chain_op(sc.ST_OP_MAXPOOL, 0, 0, _pool_desc(1, 64, 8, 8, 1))) == sc.ST_OK
    assert status(sc.make_chain_op(sc.ST_OP_MAXPOOL, 0, 0, _pool_desc(1, 12, 8, 8, 1))) == sc.ST_ERR_UNSUPPORTED     # C not a vector multiple
    p = _pool_desc(1, 64, 8, 8, 1)
    p.K = 32
    assert status(sc.make_chain_op(sc.ST_OP_MAXPOOL, 0, 0, p)) == sc.ST_ERR_INVALID_ARG
    p = _pool_desc(1, 64, 8, 8, 1)
    p.pad = 3
    assert status(sc.make_chain_op(sc.ST_OP_MAXPOOL, 0, 0, p)) == sc.ST_ERR_INVALID_ARG
