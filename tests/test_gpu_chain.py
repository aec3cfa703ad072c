"""The chain (one persistent launch over every tenant's whole sequence of layers) on the GPU, through the C ABI.

Parity against the fp64 oracle is teacher-forced per layer, as for the layer-by-layer launches: the stack is laid
out with a buffer of its own for every layer's output, so that after the ONE launch every layer's inputs (exactly
what the kernel read) and outputs are still there to be downloaded and compared element by element."""
import numpy as np
import pytest

from paper_1901_00041_amd import st_conv as sc
from paper_1901_00041_amd import synth
from paper_1901_00041_amd.synth import ConvShape

pytestmark = pytest.mark.gpu


def _nchw(t):
    return t.detach().to("cpu").double().numpy().transpose(0, 3, 1, 2)


def _check_every_layer(stack, tenants, what):
    from oracle import oracle
    worst = 0.0
    for st in stack.steps:
        s = st.shape
        for t in tenants:
            x = _nchw(stack.view(st.src, t, s.N, s.H, s.W, s.C))
            r = _nchw(stack.view(st.res, t, s.N, s.P, s.Q, s.K)) if st.res is not None else None
            ref = oracle.conv_layer(x, synth.gen_weight(5, t, st.index, s, 2.0), s.stride, s.pad, r, st.relu)
            got = _nchw(stack.view(st.dst, t, s.N, s.P, s.Q, s.K))
            err = np.abs(got - ref)
            assert np.isfinite(got).all() and (err <= 1e-2 * (np.abs(ref) + 1.0)).all(), \
                f"{what}: step {st.index} {st.name} tenant {t}: max err {err.max():.3e}"
            worst = max(worst, float((err / (np.abs(ref) + 1.0)).max()))
            if st.pool_after:
                p = (s.P + 2 - 3) // 2 + 1
                pooled = _nchw(stack.view(st.pool_dst, t, s.N, p, p, s.K))
                assert np.array_equal(pooled, oracle.maxpool2d(got, 3, 2, 1)), f"{what}: max-pool mismatch, tenant {t}"
    return worst


@pytest.mark.parametrize("target_items", [0, 256])
def test_chain_full_size_every_layer_every_element(target_items):
    """The benchmarked configuration (8 tenants x 53 layers + max-pool) as one launch: every output element of every
    layer of every tenant against the oracle, teacher-forced."""
    import torch
    from paper_1901_00041_amd.stack import ResNetStack
    n_tenants = 8
    stack = ResNetStack(n_tenants=n_tenants, unique_buffers=True,
                        plan_opts=sc.plan_opts(target_items=target_items) if target_items else None)
    stack.build_chain()
    info = stack.chain.info()
    assert info.n_sequences == n_tenants and info.n_ops == n_tenants * 54 and info.flops == n_tenants * 8174272512
    assert 0 < info.workgroups <= 1024
    stack.run("fused_chain")
    torch.cuda.synchronize()
    assert not stack.chain.aborted()
    worst = _check_every_layer(stack, range(n_tenants), f"chain target_items={target_items}")
    print(f"chain, target_items={target_items}: worst relative error {worst:.3e}; {info.n_items} queue entries, {info.workgroups} workgroups")


@pytest.mark.parametrize("chain_queues", [0, 1])
def test_chain_matches_layer_launches_bitwise_on_reused_buffers(chain_queues):
    """Both queue layouts (0: the default, one queue per XCD for these 8 sequences; 1: one queue for the whole chip,
    where producers and consumers sit on different XCDs).  The benchmark's own buffer layout (a handful of activation buffers reused all through the network): the chain's
    dependency order must cover every overwrite.  Same tiles per stage as the layer-by-layer plans, so every tenant's
    network output is bitwise the layer-by-layer one; 60 passes in a row give the same bits, two of them after a pass
    that was forced to give up."""
    import torch
    from paper_1901_00041_amd.stack import ResNetStack
    n_tenants = 8
    stack = ResNetStack(n_tenants=n_tenants)
    last = stack.steps[-1]
    s = last.shape
    stack.run("fused")
    torch.cuda.synchronize()
    want = stack.buf[last.dst].clone()
    assert float(want.float().abs().max()) > 0

    def scrub():
        for i, b in stack.buf.items():
            if i != 0:
                b.zero_()

    scrub()
    stack.build_chain(chain_queues)
    assert stack.chain.info().n_queues == (8 if chain_queues == 0 else 1)
    for rep in range(60):
        stack.run("fused_chain")
        if rep % 10 == 0:
            torch.cuda.synchronize()
            assert torch.equal(stack.buf[last.dst], want), f"pass {rep}"
            scrub()
    torch.cuda.synchronize()
    assert torch.equal(stack.buf[last.dst], want)
    assert not stack.chain.aborted()
    # a pass that gives up: with a zero wait limit the first dependency that is not yet satisfied abandons the pass;
    # the kernel exits by itself, the flag says so, and the next passes are right again
    stack.chain.set_wait_limit_us(0)
    scrub()
    stack.run("fused_chain")
    torch.cuda.synchronize()
    assert stack.chain.aborted()
    assert not stack.chain.aborted()              # reading the flag clears it
    stack.chain.set_wait_limit_us(100000)
    for _ in range(2):
        scrub()
        stack.run("fused_chain")
        torch.cuda.synchronize()
        assert torch.equal(stack.buf[last.dst], want)
    assert not stack.chain.aborted()


def test_chain_mixed_small_ops():
    """Two sequences of unequal length with fp32 and 16-bit layers, a residual, a filter count that is not a multiple of
    8 (the epilogue with plain stores, also reading a residual), channel counts that take element-wise gathers, a max-pool
    in the middle and two independent ops in one stage, with one queue and with queues per XCD: every op against the
    oracle on the tensors it read."""
    import torch
    from oracle import oracle
    from tests import helpers
    dev = "cuda"

    def tensor(shape, dtype):
        return torch.full(shape, float("nan"), dtype=helpers.torch_dtype(dtype), device=dev)

    specs = [  # (sequence, stage, ConvShape, src key, dst key, residual key, relu)
        (0, 0, ConvShape(2, 16, 9, 11, 40, 3, 3, 1, 1, "bf16", "bf16"), "in0", "a", None, True),
        (0, 1, ConvShape(2, 40, 9, 11, 24, 1, 1, 1, 0, "bf16", "bf16"), "a", "b", None, False),
        (0, 1, ConvShape(2, 40, 9, 11, 64, 3, 3, 2, 1, "bf16", "bf16"), "a", "c", None, True),
        (0, 3, ConvShape(2, 24, 9, 11, 40, 3, 3, 1, 1, "bf16", "bf16"), "b", "d", "a", True),
        (1, 0, ConvShape(1, 12, 10, 10, 20, 3, 3, 1, 1, "f32", "f32"), "in1", "e", None, True),     # 20 filters: plain stores
        (1, 2, ConvShape(1, 20, 10, 10, 36, 3, 3, 1, 1, "f32", "f32"), "e", "f", None, False),
        (1, 4, ConvShape(1, 36, 5, 5, 16, 1, 1, 1, 0, "f32", "f32"), "fp", "g", None, True),
        # element-wise gathers and the plain-store epilogue reading a residual, fp32 and 16-bit
        (1, 5, ConvShape(1, 16, 5, 5, 20, 3, 3, 1, 1, "f32", "f32"), "g", "h", None, False),
        (1, 6, ConvShape(1, 20, 5, 5, 20, 3, 3, 1, 1, "f32", "f32"), "h", "i", "h", True),
        (0, 4, ConvShape(2, 40, 9, 11, 12, 1, 1, 1, 0, "bf16", "bf16"), "d", "j", None, False),
        (0, 5, ConvShape(2, 12, 9, 11, 12, 3, 3, 1, 1, "bf16", "bf16"), "j", "k", "j", True),
    ]
    bufs = {"in0": helpers.to_device_nhwc(synth.gen_input(98, 0, 0, specs[0][2]), "bf16"),
            "in1": helpers.to_device_nhwc(synth.gen_input(98, 1, 0, specs[4][2]), "f32"),
            "fp": tensor((1, 5, 5, 36), "f32")}
    weights, ops, keep = [], [], []
    for i, (q, stage, s, src, dst, res, relu) in enumerate(specs):
        w = synth.gen_weight(98, i, 0, s, 2.0)
        dw = helpers.to_device_nhwc(w, s.dtype)
        weights.append(w)
        bufs[dst] = tensor((s.N, s.P, s.Q, s.K), s.out_dtype)
        epi = (sc.ST_EPI_RELU if relu else 0) | (sc.ST_EPI_RESIDUAL if res else 0)
        d = sc.make_desc(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, s.dtype, s.out_dtype, bufs[src], dw, bufs[dst],
                         bufs[res] if res else None, epi)
        ops.append(sc.make_chain_op(sc.ST_OP_CONV, q, stage, d))
        keep.append(dw)
    pool = sc.make_desc(1, 36, 10, 10, 36, 3, 3, 2, 1, "f32", "f32", bufs["f"], None, bufs["fp"])
    ops.append(sc.make_chain_op(sc.ST_OP_MAXPOOL, 1, 3, pool))
    # one queue for the chip (two sequences), then queues per XCD forced (completion flags, exclusive/shared queues)
    for opts in (None, sc.plan_opts(tile_cfg=4, split_k=2), sc.plan_opts(tile_cfg=6, split_k=3),
                 sc.plan_opts(chain_queues=2), sc.plan_opts(tile_cfg=4, split_k=2, chain_queues=2), sc.plan_opts(tile_cfg=5, split_k=3, chain_queues=2)):
        for k, b in bufs.items():
            if not k.startswith("in"):
                b.fill_(float("nan"))
        chain = sc.Chain(ops, opts, keep=[bufs, keep])
        assert chain.info().n_queues == (8 if opts is not None and opts.chain_queues == 2 else 1)
        for _ in range(3):
            chain.run()
        torch.cuda.synchronize()
        assert not chain.aborted()
        for i, (q, stage, s, src, dst, res, relu) in enumerate(specs):
            ref = oracle.conv_layer(_nchw(bufs[src]), weights[i], s.stride, s.pad, _nchw(bufs[res]) if res else None, relu)
            got = _nchw(bufs[dst])
            tol = helpers.tolerance(s, ref)
            err = np.abs(got - ref)
            assert np.isfinite(got).all() and (err <= tol).all(), f"op {i} opts {opts and (opts.tile_cfg, opts.split_k, opts.chain_queues)}: max err {err.max():.3e}"
        assert np.array_equal(_nchw(bufs["fp"]), oracle.maxpool2d(_nchw(bufs["f"]), 3, 2, 1))


def test_chain_sixteen_sequences_on_pingpong_buffers():
    """Sixteen sequences (two per XCD) of four dependent layers that write back and forth between two buffers (every
    stage overwrites what the stage before it read), sizes differing per sequence: many passes, each bitwise equal to
    the same layers run stage by stage as ordinary fused launches."""
    import torch
    from tests import helpers
    n_seq, n_stage = 16, 4
    rng = np.random.default_rng(7)
    seqs = []
    for q in range(n_seq):
        C = int(rng.choice([16, 32, 64]))
        H, W = int(rng.integers(7, 15)), int(rng.integers(7, 15))
        s = ConvShape(int(rng.integers(1, 3)), C, H, W, C, 3, 3, 1, 1, "bf16", "bf16")
        x = helpers.to_device_nhwc(synth.gen_input(97, q, 0, s), "bf16")
        a, b = torch.zeros_like(x), torch.zeros_like(x)
        ws = [helpers.to_device_nhwc(synth.gen_weight(97, q, l, s, 2.0), "bf16") for l in range(n_stage)]
        seqs.append((s, x, a, b, ws))
    stage_descs = []
    for l in range(n_stage):
        descs = []
        for (s, x, a, b, ws) in seqs:
            src = x if l == 0 else (a if l % 2 == 1 else b)
            dst = a if l % 2 == 0 else b
            descs.append(sc.make_desc(s.N, s.C, s.H, s.W, s.K, 3, 3, 1, 1, "bf16", "bf16", src, ws[l], dst, None, sc.ST_EPI_RELU))
        stage_descs.append(descs)
    plans = [sc.st_conv_plan(d, None, keep=[seqs]) for d in stage_descs]
    for p in plans:
        sc.st_conv_run(p)
    torch.cuda.synchronize()
    want = [(a.clone(), b.clone()) for (_, _, a, b, _) in seqs]
    ops = [sc.make_chain_op(sc.ST_OP_CONV, q, l, stage_descs[l][q]) for l in range(n_stage) for q in range(n_seq)]
    chain = sc.Chain(ops, None, keep=[seqs])
    info = chain.info()
    assert info.n_queues == 8 and info.n_sequences == n_seq
    for rep in range(20):
        if rep % 5 == 0:
            for (_, _, a, b, _) in seqs:
                a.zero_(); b.zero_()
        chain.run()
        if rep % 5 == 4:
            torch.cuda.synchronize()
            for q, (_, _, a, b, _) in enumerate(seqs):
                assert torch.equal(a, want[q][0]) and torch.equal(b, want[q][1]), f"pass {rep}, sequence {q}"
    assert not chain.aborted()


@pytest.mark.parametrize("chain_queues", [0, 1])
def test_chain_with_fewer_workgroups_than_planned(chain_queues):
    """The one-queue form completes with any number of workgroups.  The column form needs a workgroup for every column
    in use: launched with one workgroup per compute unit only (nobody draws the shared columns), the dependants of the
    undone entries give up after the wait limit, the kernel exits by itself, the pass is reported as abandoned, and
    the next full-size pass is right again."""
    import torch
    from paper_1901_00041_amd.stack import ResNetStack
    stack = ResNetStack(n_tenants=8)
    last = stack.steps[-1]
    stack.run("fused")
    torch.cuda.synchronize()
    want = stack.buf[last.dst].clone()
    stack.build_chain(chain_queues)
    chain = stack.chain
    planned = chain.info().workgroups
    with pytest.raises(sc.StError):
        chain.set_workgroups(planned + 1)

    def scrub():
        for i, b in stack.buf.items():
            if i != 0:
                b.zero_()

    scrub()
    if chain_queues == 1:
        chain.set_workgroups(64)
        stack.run("fused_chain")
        torch.cuda.synchronize()
        assert not chain.aborted() and torch.equal(stack.buf[last.dst], want)
    else:
        assert planned == 512
        chain.set_workgroups(256)
        chain.set_wait_limit_us(2000)
        stack.run("fused_chain")
        torch.cuda.synchronize()
        assert chain.aborted()
        chain.set_workgroups(0)
        chain.set_wait_limit_us(100000)
        scrub()
        stack.run("fused_chain")
        torch.cuda.synchronize()
        assert not chain.aborted() and torch.equal(stack.buf[last.dst], want)
