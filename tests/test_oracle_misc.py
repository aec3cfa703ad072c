"""Pins of the oracle's element-wise pieces: bfloat16 rounding, max-pool, ReLU, layer composition."""
import numpy as np
import pytest

from oracle import oracle


def _all_bf16_values():
    bits = np.arange(65536, dtype=np.uint32) << np.uint32(16)
    return bits.view(np.float32)


def test_round_bf16_every_pattern_is_a_fixed_point():
    with np.errstate(invalid="ignore"):
        v = _all_bf16_values().astype(np.float64)
    finite = np.isfinite(v)
    r = oracle.round_bf16(v[finite])
    assert np.array_equal(r, v[finite])
    assert np.array_equal(np.signbit(r), np.signbit(v[finite]))
    inf = oracle.round_bf16(np.array([np.inf, -np.inf]))
    assert inf[0] == np.inf and inf[1] == -np.inf and np.isnan(oracle.round_bf16(np.array([np.nan]))[0])


def test_round_bf16_ties_and_neighbours():
    u = 2.0 ** -7          # spacing in [1,2)
    cases = {1.0 + u / 2: 1.0, 1.0 + 3 * u / 2: 1.0 + 2 * u, 1.0 + u / 2 + 1e-9: 1.0 + u,
             -(1.0 + u / 2): -1.0, 1.0 + u / 2 - 1e-9: 1.0, 255.5: 256.0, 3.0e38: 226 * 2.0 ** 120}
    for v, want in cases.items():
        got = oracle.round_bf16(np.array([v]))[0]
        assert got == want, (v, got, want)
    big = float(np.float32(3.3895314e38))      # largest finite bfloat16
    assert oracle.round_bf16(np.array([big]))[0] == big
    assert oracle.round_bf16(np.array([3.4e38]))[0] == np.inf
    # subnormal spacing is 2^-133
    assert oracle.round_bf16(np.array([2.0 ** -133 * 2.5]))[0] == 2.0 ** -133 * 2
    assert oracle.round_bf16(np.array([2.0 ** -133 * 3.5]))[0] == 2.0 ** -133 * 4


def test_round_bf16_against_library_cast():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(7)
    a = (rng.standard_normal(1_000_000) * np.exp(rng.uniform(-20, 20, 1_000_000))).astype(np.float32)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(oracle.round_bf16(a.astype(np.float64)), want)


def test_maxpool_brute_force_and_library():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(11)
    x = rng.uniform(-1, 1, size=(2, 3, 9, 8))
    y = oracle.maxpool2d(x, 3, 2, 1)
    assert y.shape == (2, 3, 5, 4)
    xp = np.full((2, 3, 11, 10), -np.inf)
    xp[:, :, 1:10, 1:9] = x
    for p in range(5):
        for q in range(4):
            assert np.array_equal(y[:, :, p, q], xp[:, :, 2 * p:2 * p + 3, 2 * q:2 * q + 3].max(axis=(2, 3)))
    want = torch.nn.functional.max_pool2d(torch.from_numpy(x), 3, 2, 1).numpy()
    assert np.array_equal(y, want)
    assert oracle.maxpool2d(np.zeros((1, 64, 112, 112))).shape == (1, 64, 56, 56)


def test_relu_and_layer_composition():
    rng = np.random.default_rng(3)
    x, w = rng.uniform(-1, 1, (1, 4, 5, 5)), rng.uniform(-1, 1, (6, 4, 3, 3))
    res = rng.uniform(-1, 1, (1, 6, 5, 5))
    base = oracle.conv2d(x, w, 1, 1)
    assert np.array_equal(oracle.relu(np.array([-1.0, 0.0, 2.5])), np.array([0.0, 0.0, 2.5]))
    assert np.array_equal(oracle.conv_layer(x, w, 1, 1), base)
    assert np.array_equal(oracle.conv_layer(x, w, 1, 1, residual=res), base + res)
    got = oracle.conv_layer(x, w, 1, 1, residual=res, apply_relu=True)
    assert np.array_equal(got, np.where(base + res > 0, base + res, 0.0))
    # ReLU comes after the residual add, not before
    assert not np.array_equal(got, np.maximum(base, 0) + res)
