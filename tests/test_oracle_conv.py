"""Pins of the fp64 convolution oracle against what the definition and the paper fix (CPU only).

Each test is chosen so that one plausible mistake (flipped filter, transposed operand, wrong stride
or padding offset, dropped tap, wrong channel pairing) fails it.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import oracle

RNG = np.random.default_rng(20190100041)


def _rand(*shape):
    return RNG.uniform(-1.0, 1.0, size=shape)


def im2col_reference(x, w, stride, pad):
    """Second, differently structured routine: explicit zero-padded copy, materialised patch matrix,
    then one matrix product (the lowering Section 4.1 names)."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad))
    xp[:, :, pad:pad + H, pad:pad + W] = x
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    cols = np.empty((N * P * Q, C * R * S))
    row = 0
    for n in range(N):
        for p in range(P):
            for q in range(Q):
                cols[row] = xp[n, :, p * stride:p * stride + R, q * stride:q * stride + S].reshape(-1)
                row += 1
    y = cols @ w.reshape(K, -1).T                     # (N*P*Q, K)
    return y.reshape(N, P, Q, K).transpose(0, 3, 1, 2)


def test_hand_computed_3x3():
    # Worked by hand: Sobel-like filter, pad 1.  y[p,q] = sum_r rw[r]*(x[p-1+r,q-1]-x[p-1+r,q+1]),
    # rw=[1,2,1], zeros outside.  A flipped filter negates every entry; a transposed one differs.
    x = np.arange(1.0, 10.0).reshape(1, 1, 3, 3)
    w = np.array([[1.0, 0.0, -1.0], [2.0, 0.0, -2.0], [1.0, 0.0, -1.0]]).reshape(1, 1, 3, 3)
    want = np.array([[-9.0, -6.0, 9.0], [-20.0, -8.0, 20.0], [-21.0, -6.0, 21.0]])
    assert np.array_equal(oracle.conv2d(x, w, 1, 1)[0, 0], want)


def test_hand_computed_stride2_two_channels():
    # 2 channels, 1x2 filter, stride 2, no padding, 1x4 image: y[q] = sum_c x[c,2q]*w[c,0]+x[c,2q+1]*w[c,1]
    x = np.array([[1.0, 2.0, 3.0, 4.0], [10.0, 20.0, 30.0, 40.0]]).reshape(1, 2, 1, 4)
    w = np.array([[1.0, -1.0], [0.5, 0.25]]).reshape(1, 2, 1, 2)
    assert oracle.conv2d(x, w, 2, 0).reshape(-1).tolist() == [1 - 2 + 5 + 5, 3 - 4 + 15 + 10]


def test_brute_force_grid_against_im2col():
    worst = 0.0
    for (R, S, stride, pad) in itertools.product((1, 2, 3), (1, 2, 3), (1, 2), (0, 1, 2)):
        for (N, C, H, W, K) in ((1, 1, 3, 3, 1), (2, 3, 4, 3, 2), (1, 4, 3, 4, 3), (3, 2, 4, 4, 4)):
            if H + 2 * pad < R or W + 2 * pad < S:
                continue
            x, w = _rand(N, C, H, W), _rand(K, C, R, S)
            got = oracle.conv2d(x, w, stride, pad)
            want = im2col_reference(x, w, stride, pad)
            assert got.shape == want.shape
            worst = max(worst, np.abs(got - want).max())
    assert worst < 1e-13


def test_paper_shapes_derived_dims():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_gemm_shapes.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for name, M, N, K, *desc in rows:
        d = oracle.dims(*map(int, desc))
        if name == "matvec_rnn":
            assert sorted((d["M"], d["Ngemm"])) == sorted((int(M), int(N))) and d["Kgemm"] == int(K)
        else:
            assert (d["M"], d["Ngemm"], d["Kgemm"]) == (int(M), int(N), int(K))
        assert d["flops"] == 2 * int(M) * int(N) * int(K)
    assert oracle.dims(1, 128, 16, 16, 128, 3, 3, 1, 1)["flops"] == 75497472


def test_output_size_floor_rule():
    assert oracle.out_dim(224, 7, 2, 3) == 112       # ResNet stem
    assert oracle.out_dim(112, 3, 2, 1) == 56        # its max-pool
    assert oracle.out_dim(7, 3, 2, 0) == 3 and oracle.out_dim(8, 3, 2, 0) == 3
    assert oracle.out_dim(2, 3, 1, 0) == 0


def test_1x1_is_a_matrix_product_textbook_loop():
    N, C, H, W, K = 2, 5, 3, 4, 6
    x, w = _rand(N, C, H, W), _rand(K, C, 1, 1)
    y = oracle.conv2d(x, w)
    for n in range(N):
        for h in range(H):
            for v in range(W):
                for k in range(K):
                    acc = 0.0
                    for c in range(C):
                        acc += x[n, c, h, v] * w[k, c, 0, 0]
                    assert abs(y[n, k, h, v] - acc) < 1e-14


@pytest.mark.parametrize("C,K,H", [(256, 256, 16), (512, 512, 1)])
def test_1x1_paper_shapes_against_matmul(C, K, H):
    # Table 1: square 256^3 and matrix-vector (512,1,512) as 1x1 convolutions.
    x, w = _rand(1, C, H, H), _rand(K, C, 1, 1)
    y = oracle.conv2d(x, w)
    want = (w.reshape(K, C) @ x.reshape(C, H * H)).reshape(1, K, H, H)
    assert np.abs(y - want).max() < 1e-12


def test_section41_example_against_im2col_product():
    x, w = _rand(1, 128, 16, 16), _rand(128, 128, 3, 3) / 34.0
    y = oracle.conv2d(x, w, 1, 1)
    want = im2col_reference(x, w, 1, 1)
    assert y.shape == (1, 128, 16, 16) and np.abs(y - want).max() < 1e-12


@pytest.mark.parametrize("R", [1, 3, 5])
def test_delta_filter_is_identity(R):
    C = 3
    x = _rand(2, C, 6, 5)
    w = np.zeros((C, C, R, R))
    for c in range(C):
        w[c, c, R // 2, R // 2] = 1.0
    assert np.array_equal(oracle.conv2d(x, w, 1, R // 2), x)


def test_shifted_delta_shifts_with_zero_border():
    x = _rand(1, 1, 5, 6)
    w = np.zeros((1, 1, 3, 3))
    w[0, 0, 0, 2] = 1.0          # tap at r=0 (one row up), s=2 (one column right)
    y = oracle.conv2d(x, w, 1, 1)[0, 0]
    want = np.zeros((5, 6))
    want[1:, :-1] = x[0, 0, :-1, 1:]     # y[p,q] = x[p-1, q+1]
    assert np.array_equal(y, want)


def test_linearity_in_input_and_in_weights():
    x1, x2, w1, w2 = _rand(2, 4, 7, 6), _rand(2, 4, 7, 6), _rand(5, 4, 3, 2), _rand(5, 4, 3, 2)
    a, b = 0.75, -1.5
    lhs = oracle.conv2d(a * x1 + b * x2, w1, 2, 1)
    rhs = a * oracle.conv2d(x1, w1, 2, 1) + b * oracle.conv2d(x2, w1, 2, 1)
    assert np.abs(lhs - rhs).max() <= 1e-12 * (1 + np.abs(rhs).max())
    lhs = oracle.conv2d(x1, a * w1 + b * w2, 2, 1)
    rhs = a * oracle.conv2d(x1, w1, 2, 1) + b * oracle.conv2d(x1, w2, 2, 1)
    assert np.abs(lhs - rhs).max() <= 1e-12 * (1 + np.abs(rhs).max())


def test_all_ones_input_gives_weight_sums():
    K, C, R, S = 4, 3, 3, 3
    w = _rand(K, C, R, S)
    x = np.ones((1, C, 6, 7))
    y0 = oracle.conv2d(x, w, 1, 0)
    full = w.sum(axis=(1, 2, 3))
    assert np.abs(y0 - full[None, :, None, None]).max() < 1e-13
    y1 = oracle.conv2d(x, w, 1, 1)
    assert np.abs(y1[:, :, 1:-1, 1:-1] - full[None, :, None, None]).max() < 1e-13
    # corner (0,0): only taps r,s in {1,2} are inside; top edge: r in {1,2}, all s
    assert np.abs(y1[0, :, 0, 0] - w[:, :, 1:, 1:].sum(axis=(1, 2, 3))).max() < 1e-13
    assert np.abs(y1[0, :, 0, 3] - w[:, :, 1:, :].sum(axis=(1, 2, 3))).max() < 1e-13
    assert np.abs(y1[0, :, -1, -1] - w[:, :, :2, :2].sum(axis=(1, 2, 3))).max() < 1e-13


def test_against_library_float64_convolution():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    cases = [(2, 8, 9, 11, 6, 3, 3, 1, 1), (1, 3, 23, 17, 8, 7, 7, 2, 3), (3, 16, 7, 7, 12, 1, 1, 1, 0),
             (1, 5, 10, 12, 4, 3, 2, 2, 0), (2, 4, 8, 8, 4, 1, 1, 2, 0), (1, 6, 5, 5, 3, 5, 5, 1, 2)]
    for (N, C, H, W, K, R, S, st, pd) in cases:
        x, w = _rand(N, C, H, W), _rand(K, C, R, S)
        want = F.conv2d(torch.from_numpy(x), torch.from_numpy(w), stride=st, padding=pd).numpy()
        got = oracle.conv2d(x, w, st, pd)
        assert got.shape == want.shape and np.abs(got - want).max() < 1e-12


def test_points_equal_full_result():
    x, w = _rand(2, 6, 9, 8), _rand(5, 6, 3, 3)
    y = oracle.conv2d(x, w, 2, 1)
    idx = np.array([(n, k, p, q) for n in range(2) for k in (0, 4) for p in (0, 2, 4) for q in (0, 3)], dtype=np.int32)
    pts = oracle.conv2d_points(x, w, idx, 2, 1)
    assert np.array_equal(pts, y[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]])


def test_planted_mistakes_are_caught():
    """The pins above discriminate: each classic mistake, planted in a copy of the reference routine,
    changes the hand-computed example or the shifted-delta case."""
    x = np.arange(1.0, 10.0).reshape(1, 1, 3, 3)
    w = np.array([[1.0, 0.0, -1.0], [2.0, 0.0, -2.0], [1.0, 0.0, -1.0]]).reshape(1, 1, 3, 3)
    good = oracle.conv2d(x, w, 1, 1)
    flipped = oracle.conv2d(x, w[:, :, ::-1, ::-1], 1, 1)
    transposed = oracle.conv2d(x, w.transpose(0, 1, 3, 2), 1, 1)
    assert not np.array_equal(good, flipped) and not np.array_equal(good, transposed)
