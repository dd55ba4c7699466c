"""Pins for the fp64 convolution oracle (CPU only).

The oracle is checked against things other than itself: hand-computed cases,
closed forms (padding counts, identity filter), special cases that reduce to a
plain matrix product (numpy's matmul), torch's CPU float64 conv2d and autograd
(a library routine for the same definition), the adjoint identities, finite
differences, and the tensor sizes the paper prints for AlexNet.
"""
import os

import numpy as np
import pytest
import torch

import oracle

RNG = np.random.default_rng(1234)

# (N, C, H, W, K, R, S, stride, pad)
SHAPES = [
    (2, 3, 7, 9, 4, 3, 3, (1, 1), (1, 1)),
    (1, 2, 8, 8, 3, 3, 3, (2, 2), (1, 1)),
    (2, 3, 11, 13, 2, 5, 5, (1, 1), (2, 2)),
    (1, 3, 23, 19, 4, 11, 11, (4, 4), (0, 0)),
    (2, 4, 9, 17, 3, 1, 7, (1, 1), (0, 3)),
    (2, 4, 17, 9, 3, 7, 1, (1, 1), (3, 0)),
    (3, 5, 6, 6, 7, 1, 1, (1, 1), (0, 0)),
    (2, 4, 8, 8, 6, 1, 1, (2, 2), (0, 0)),
    (1, 2, 9, 9, 2, 3, 3, (2, 2), (0, 0)),
    (1, 2, 10, 7, 3, 3, 2, (2, 1), (1, 0)),
    (1, 1, 5, 6, 1, 2, 3, (3, 2), (1, 2)),
]


def _rand(*shape):
    return RNG.standard_normal(shape)


def test_hand_case_2x2_filter():
    # x = 1..9 on a 3x3 grid, filter [[1,2],[3,4]], stride 1, no padding.
    x = np.arange(1.0, 10.0).reshape(1, 1, 3, 3)
    w = np.array([[1.0, 2.0], [3.0, 4.0]]).reshape(1, 1, 2, 2)
    y = oracle.conv2d_fwd(x, w)
    # by hand: 1*1+2*2+3*4+4*5 = 37, 1*2+2*3+3*5+4*6 = 47, 67, 77
    assert y.shape == (1, 1, 2, 2)
    assert y.ravel().tolist() == [37.0, 47.0, 67.0, 77.0]


def test_no_filter_flip():
    # A filter with a single 1 at (r,s)=(0,1) shifts the image left by one
    # column under cross-correlation (it would shift right under convolution).
    x = np.arange(12.0).reshape(1, 1, 3, 4)
    w = np.zeros((1, 1, 1, 2))
    w[0, 0, 0, 1] = 1.0
    y = oracle.conv2d_fwd(x, w)
    assert np.array_equal(y[0, 0], x[0, 0, :, 1:])


def test_centre_delta_is_identity():
    x = _rand(2, 3, 6, 5)
    w = np.zeros((3, 3, 3, 3))
    for c in range(3):
        w[c, c, 1, 1] = 1.0
    assert np.array_equal(oracle.conv2d_fwd(x, w, pad=(1, 1)), x)


def test_padding_counts():
    # all-ones image and 3x3 all-ones filter, pad 1: the output counts the taps
    # inside the image: 4 at corners, 6 on edges, 9 inside.
    y = oracle.conv2d_fwd(np.ones((1, 1, 5, 6)), np.ones((1, 1, 3, 3)), pad=(1, 1))[0, 0]
    want = np.full((5, 6), 9.0)
    want[0, :] = want[-1, :] = 6.0
    want[:, 0] = want[:, -1] = 6.0
    want[0, 0] = want[0, -1] = want[-1, 0] = want[-1, -1] = 4.0
    assert np.array_equal(y, want)


def test_stride2_hand_case():
    # 1x1x5x5 ramp, 3x3 ones, stride 2, pad 0 -> 2x2 sums of 3x3 blocks.
    x = np.arange(25.0).reshape(1, 1, 5, 5)
    y = oracle.conv2d_fwd(x, np.ones((1, 1, 3, 3)), stride=(2, 2))[0, 0]
    want = np.array([[x[0, 0, i:i + 3, j:j + 3].sum() for j in (0, 2)] for i in (0, 2)])
    assert np.array_equal(y, want)


def test_asymmetric_1x7_hand_case():
    # 1x7 ones filter with pad (0,3): running sum of up to 7 neighbours in a row.
    x = np.arange(1.0, 11.0).reshape(1, 1, 1, 10)
    y = oracle.conv2d_fwd(x, np.ones((1, 1, 1, 7)), pad=(0, 3))[0, 0, 0]
    want = [sum(v for j, v in enumerate(range(1, 11)) if abs(j - i) <= 3) for i in range(10)]
    assert y.tolist() == [float(v) for v in want]


def test_1x1_is_matmul():
    x, w = _rand(3, 5, 4, 6), _rand(7, 5, 1, 1)
    y = oracle.conv2d_fwd(x, w)
    want = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0], x)
    np.testing.assert_allclose(y, want, rtol=1e-13, atol=1e-13)


def test_filter_equals_stride_is_block_matmul():
    # R = S = stride, no padding: non-overlapping patches, one matmul.
    N, C, K, B = 2, 3, 4, 2
    x, w = _rand(N, C, 6, 8), _rand(K, C, B, B)
    y = oracle.conv2d_fwd(x, w, stride=(B, B))
    patches = x.reshape(N, C, 3, B, 4, B).transpose(0, 2, 4, 1, 3, 5).reshape(N, 3, 4, C * B * B)
    want = (patches @ w.reshape(K, -1).T).transpose(0, 3, 1, 2)
    np.testing.assert_allclose(y, want, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("shape", SHAPES)
def test_against_torch_cpu_float64(shape):
    N, C, H, W, K, R, S, stride, pad = shape
    x, w = _rand(N, C, H, W), _rand(K, C, R, S)
    xt = torch.from_numpy(x).requires_grad_(True)
    wt = torch.from_numpy(w).requires_grad_(True)
    yt = torch.nn.functional.conv2d(xt, wt, stride=stride, padding=pad)
    y = oracle.conv2d_fwd(x, w, stride, pad)
    assert y.shape == tuple(yt.shape)
    np.testing.assert_allclose(y, yt.detach().numpy(), rtol=1e-12, atol=1e-12)
    dy = _rand(*y.shape)
    yt.backward(torch.from_numpy(dy))
    np.testing.assert_allclose(oracle.conv2d_bwd_data(dy, w, x.shape, stride, pad),
                               xt.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.conv2d_bwd_filter(x, dy, w.shape, stride, pad),
                               wt.grad.numpy(), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("shape", SHAPES)
def test_adjoint_identities(shape):
    N, C, H, W, K, R, S, stride, pad = shape
    x, w = _rand(N, C, H, W), _rand(K, C, R, S)
    y = oracle.conv2d_fwd(x, w, stride, pad)
    dy = _rand(*y.shape)
    lhs = float((y * dy).sum())
    a = float((x * oracle.conv2d_bwd_data(dy, w, x.shape, stride, pad)).sum())
    b = float((w * oracle.conv2d_bwd_filter(x, dy, w.shape, stride, pad)).sum())
    scale = max(1.0, abs(lhs))
    assert abs(lhs - a) <= 1e-11 * scale
    assert abs(lhs - b) <= 1e-11 * scale


def test_finite_differences():
    N, C, H, W, K, R, S, stride, pad = 1, 2, 6, 5, 3, 3, 3, (2, 1), (1, 1)
    x, w = _rand(N, C, H, W), _rand(K, C, R, S)
    dy = _rand(*oracle.conv2d_fwd(x, w, stride, pad).shape)

    def loss(xx, ww):
        return float((oracle.conv2d_fwd(xx, ww, stride, pad) * dy).sum())

    dx = oracle.conv2d_bwd_data(dy, w, x.shape, stride, pad)
    dw = oracle.conv2d_bwd_filter(x, dy, w.shape, stride, pad)
    h = 1e-3  # the loss is bilinear, so central differences are exact up to rounding
    for idx in [(0, 0, 0, 0), (0, 1, 3, 2), (0, 1, 5, 4), (0, 0, 2, 3)]:
        e = np.zeros_like(x)
        e[idx] = h
        fd = (loss(x + e, w) - loss(x - e, w)) / (2 * h)
        assert abs(fd - dx[idx]) <= 1e-9 * max(1.0, abs(fd))
    for idx in [(0, 0, 0, 0), (2, 1, 2, 2), (1, 0, 1, 2)]:
        e = np.zeros_like(w)
        e[idx] = h
        fd = (loss(x, w + e) - loss(x, w - e)) / (2 * h)
        assert abs(fd - dw[idx]) <= 1e-9 * max(1.0, abs(fd))


def test_linearity_and_translation():
    x1, x2, w = _rand(1, 2, 8, 8), _rand(1, 2, 8, 8), _rand(3, 2, 3, 3)
    y = oracle.conv2d_fwd(2.0 * x1 - 3.0 * x2, w, pad=(1, 1))
    want = 2.0 * oracle.conv2d_fwd(x1, w, pad=(1, 1)) - 3.0 * oracle.conv2d_fwd(x2, w, pad=(1, 1))
    np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-12)
    # shifting the image by (1,2) shifts interior outputs by (1,2)
    xs = np.zeros_like(x1)
    xs[:, :, 1:, 2:] = x1[:, :, :-1, :-2]
    ys = oracle.conv2d_fwd(xs, w, pad=(1, 1))
    y1 = oracle.conv2d_fwd(x1, w, pad=(1, 1))
    np.testing.assert_allclose(ys[:, :, 3:7, 4:7], y1[:, :, 2:6, 2:5], rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("shape", SHAPES[:6])
def test_point_versions_match_full(shape):
    N, C, H, W, K, R, S, stride, pad = shape
    x, w = _rand(N, C, H, W), _rand(K, C, R, S)
    y = oracle.conv2d_fwd(x, w, stride, pad)
    dy = _rand(*y.shape)
    dx = oracle.conv2d_bwd_data(dy, w, x.shape, stride, pad)
    dw = oracle.conv2d_bwd_filter(x, dy, w.shape, stride, pad)
    r = np.random.default_rng(7)
    for _ in range(8):
        n, k, p, q = (int(r.integers(0, d)) for d in y.shape)
        assert abs(oracle.conv2d_fwd_at(x, w, stride, pad, n, k, p, q) - y[n, k, p, q]) < 1e-12
        n, c, h, v = (int(r.integers(0, d)) for d in x.shape)
        assert abs(oracle.conv2d_bwd_data_at(dy, w, x.shape, stride, pad, n, c, h, v) - dx[n, c, h, v]) < 1e-12
        k, c, rr, s = (int(r.integers(0, d)) for d in w.shape)
        assert abs(oracle.conv2d_bwd_filter_at(x, dy, w.shape, stride, pad, k, c, rr, s) - dw[k, c, rr, s]) < 1e-11


@pytest.mark.parametrize("shape", SHAPES)
def test_point_list_versions_match_full(shape):
    """Every output element through the list versions (backward-data solves for the output row and
    column per tap instead of walking all of them) against the pinned full loops, on every shape of
    the list: strides 1, 2 and 4, asymmetric and zero padding."""
    N, C, H, W, K, R, S, stride, pad = shape
    x, w = _rand(N, C, H, W), _rand(K, C, R, S)
    y = oracle.conv2d_fwd(x, w, stride, pad)
    dy = _rand(*y.shape)
    dx = oracle.conv2d_bwd_data(dy, w, x.shape, stride, pad)
    dw = oracle.conv2d_bwd_filter(x, dy, w.shape, stride, pad)

    def every(shape4):
        return np.stack(np.meshgrid(*[np.arange(d) for d in shape4], indexing="ij"), -1).reshape(-1, 4)

    np.testing.assert_allclose(oracle.conv2d_fwd_points(x, w, stride, pad, every(y.shape)), y.ravel(),
                               rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.conv2d_bwd_data_points(dy, w, x.shape, stride, pad, every(x.shape)),
                               dx.ravel(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.conv2d_bwd_filter_points(x, dy, w.shape, stride, pad, every(w.shape)),
                               dw.ravel(), rtol=0, atol=1e-11)


def test_paper_alexnet_tensor_sizes():
    path = os.path.join(os.path.dirname(__file__), "golden", "alexnet_conv_output_mib.txt")
    want = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            name, val = line.split()
            want[name] = float(val)
    batch = 200
    h = oracle.out_dim(227, 0, 11, 4)          # CONV1 11x11 stride 4
    sizes = {"CONV1": batch * 96 * h * h * 4}
    h = oracle.out_dim(h, 0, 3, 2)             # POOL1 3x3 stride 2
    h = oracle.out_dim(h, 2, 5, 1)             # CONV2 5x5 pad 2
    sizes["CONV2"] = batch * 256 * h * h * 4
    h = oracle.out_dim(h, 0, 3, 2)             # POOL2
    h = oracle.out_dim(h, 1, 3, 1)             # CONV3 3x3 pad 1
    sizes["CONV3"] = batch * 384 * h * h * 4
    h = oracle.out_dim(h, 1, 3, 1)             # CONV4
    sizes["CONV4"] = batch * 384 * h * h * 4
    for name, nbytes in sizes.items():
        assert round(nbytes / 2 ** 20, 2) == want[name], (name, nbytes / 2 ** 20)
    # the oracle's own output shape follows the same rule
    y = oracle.conv2d_fwd(np.zeros((1, 1, 227, 227)), np.zeros((1, 1, 11, 11)), stride=(4, 4))
    assert y.shape == (1, 1, 55, 55)
