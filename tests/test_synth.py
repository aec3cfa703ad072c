"""Generator and workload-recipe pins (CPU)."""
import numpy as np

from paper_1901_00041_amd import synth


def test_splitmix64_published_vector():
    # Widely published outputs of splitmix64 started from state 0.
    out = synth.splitmix64(0, 3)
    assert [hex(int(v)) for v in out] == ["0xe220a8397b1dcdaf", "0x6e789e6aa1b965f4", "0x6c45d188009454f"]
    # slices are consistent with the whole
    assert np.array_equal(synth.splitmix64(0, 2, offset=1), out[1:])


def test_splitmix64_matches_scalar_reference():
    mask = (1 << 64) - 1
    s = 0x1234ABCD
    want = []
    for _ in range(5):
        s = (s + 0x9E3779B97F4A7C15) & mask
        z = s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
        want.append(z ^ (z >> 31))
    assert [int(v) for v in synth.splitmix64(0x1234ABCD, 5)] == want


def test_uniform_and_normal_moments():
    u = synth.uniform_pm1(synth.stream_state(9, 0, 0, 1), 200000)
    assert -1.0 <= u.min() and u.max() < 1.0
    assert abs(u.mean()) < 0.01 and abs(u.var() - 1.0 / 3.0) < 0.01
    g = synth.normal(synth.stream_state(9, 0, 0, 2), 200000, 0.5)
    assert abs(g.mean()) < 0.01 and abs(g.std() - 0.5) < 0.01


def test_bf16_storage_rounding_ties_to_even():
    a = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 1.0 + 2.0 ** -8 + 2.0 ** -20],
                 dtype=np.float32)
    got = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(a))
    assert got.tolist() == [1.0, 1.0, 1.015625, -1.0, 1.0078125]


def test_config3_batches():
    assert [s.N for s in synth.config_shapes(3)] == [2, 1, 4, 1, 1, 4, 2, 1]


def test_config4_descriptors():
    want = [(5, 512, 7, 7, 128, 1, 1, 1, 0), (1, 512, 56, 56, 512, 3, 3, 1, 1), (4, 64, 28, 28, 512, 1, 1, 1, 0),
            (1, 256, 56, 56, 256, 3, 3, 1, 1), (3, 256, 28, 28, 512, 1, 1, 1, 0), (1, 64, 14, 14, 64, 3, 3, 1, 1),
            (3, 128, 56, 56, 512, 1, 1, 1, 0), (2, 3, 224, 224, 64, 7, 7, 2, 3), (1, 512, 7, 7, 256, 1, 1, 1, 0),
            (4, 256, 7, 7, 256, 3, 3, 1, 1), (6, 256, 7, 7, 1024, 1, 1, 1, 0), (4, 128, 7, 7, 128, 3, 3, 1, 1),
            (2, 256, 7, 7, 1024, 1, 1, 1, 0), (3, 128, 56, 56, 128, 3, 3, 1, 1), (1, 1024, 14, 14, 64, 1, 1, 1, 0),
            (8, 3, 224, 224, 64, 7, 7, 2, 3)]
    got = [(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad) for s in synth.config_shapes(4)]
    assert got == want
    gemm = [s.gemm for s in synth.config_shapes(4)]
    assert gemm[0] == (245, 128, 512) and gemm[1] == (3136, 512, 4608) and gemm[15] == (100352, 64, 147)


def test_config_totals():
    tot = {c: sum(s.flops for s in synth.config_shapes(c)) for c in (1, 2, 3, 4)}
    assert tot[1] == 2 * 2 * 784 * 32 * 288
    assert tot[2] == 4 * 231211008
    assert abs(tot[3] / 1e9 - 3.70) < 0.01
    assert abs(tot[4] / 1e9 - 26.27) < 0.01
    by = {c: sum(s.bytes for s in synth.config_shapes(c)) for c in (1, 2, 3, 4)}
    assert abs(by[1] / 1e6 - 0.475) < 0.001
    assert abs(by[2] / 1e6 - 8.52) < 0.01
    assert abs(by[3] / 1e6 - 14.25) < 0.01
    assert abs(by[4] / 1e6 - 104.4) < 0.1


def test_resnet50_schedule_invariants():
    # Well-known facts about the standard ResNet-50: 53 convolutions; 23 454 912 convolution weights
    # (25 557 032 parameters minus the 2 049 000 of the classifier and 53 120 of batch-norm);
    # final feature map 2048 x 7 x 7 for a 224 x 224 input.
    steps = synth.resnet50_steps()
    assert len(steps) == 53
    assert sum(s.shape.K * s.shape.C * s.shape.R * s.shape.S for s in steps) == 23454912
    last = steps[-1].shape
    assert (last.K, last.P, last.Q) == (2048, 7, 7)
    assert sum(s.shape.flops for s in steps) == 8174272512
    assert len({s.shape.gemm for s in steps}) == 20
    assert sum(1 for s in steps if s.name.endswith(".proj")) == 4
    # data flow: every conv reads a buffer that was written before it
    written = {0}
    for s in steps:
        assert s.src in written and (s.res is None or s.res in written)
        written.add(s.dst)
        if s.pool_after:
            written.add(s.pool_dst)
    # stride-2 sits on the 3x3 of the first block of stages 3-5
    assert [s.name for s in steps if s.shape.stride == 2 and s.shape.R == 3] == ["s3b0.conv2", "s4b0.conv2", "s5b0.conv2"]


def test_generated_tensors_are_storage_exact_and_tenant_distinct():
    sh = synth.config_shapes(2)[3]
    w0 = synth.gen_weight(2, 0, 0, sh)
    w1 = synth.gen_weight(2, 1, 0, sh)
    assert w0.shape == (512, 512, 3, 3) and not np.array_equal(w0, w1)
    assert np.array_equal(synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(w0)).reshape(w0.shape), w0)
    assert abs(w0.std() * np.sqrt(512 * 9) - 1.0) < 0.02
    x = synth.gen_input(1, 0, 0, synth.config_shapes(1)[0])
    assert x.dtype == np.float32 and x.shape == (1, 32, 28, 28) and np.abs(x).max() < 1.0
