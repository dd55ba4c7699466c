"""Pins for the fp64 oracle of the cheap layers (ReLU, BN, max-pool), CPU only.

Checked against hand cases, closed forms and invariants, finite differences,
and torch's CPU float64 routines (library implementations of the same
definitions) -- never against the oracle's own formulas.
"""
import numpy as np
import pytest
import torch

import oracle

RNG = np.random.default_rng(99)


# ----------------------------------------------------------------- ReLU
def test_relu_hand_vector():
    x = np.array([-2.0, -1e-300, -0.0, 0.0, 1e-300, 3.5])
    assert oracle.relu_fwd(x).tolist() == [0.0, 0.0, 0.0, 0.0, 1e-300, 3.5]
    dy = np.array([1.0, 2.0, 3.0, 4.0, 5.0, 6.0])
    # gradient is 0 at x == 0 (strict gate)
    assert oracle.relu_bwd(x, dy).tolist() == [0.0, 0.0, 0.0, 0.0, 5.0, 6.0]


def test_relu_idempotent_and_mask():
    x, dy = RNG.standard_normal(1000), RNG.standard_normal(1000)
    y = oracle.relu_fwd(x)
    assert np.array_equal(oracle.relu_fwd(y), y)
    assert np.array_equal(oracle.relu_bwd(x, dy), dy * (x > 0))
    # gating on the output is equivalent to gating on the input
    assert np.array_equal(oracle.relu_bwd(y, dy), oracle.relu_bwd(x, dy))


# ----------------------------------------------------------------- BN
def test_bn_closed_forms():
    N, C, H, W = 4, 3, 5, 7
    x = RNG.standard_normal((N, C, H, W)) * np.array([0.5, 2.0, 10.0]).reshape(1, C, 1, 1) + 3.0
    gamma, beta = np.array([1.5, -0.7, 2.0]), np.array([0.1, -0.2, 4.0])
    eps = 1e-5
    y, mean, invstd = oracle.bn_fwd(x, gamma, beta, eps)
    var = x.var(axis=(0, 2, 3))  # numpy: biased
    np.testing.assert_allclose(mean, x.mean(axis=(0, 2, 3)), rtol=1e-13)
    np.testing.assert_allclose(invstd, 1.0 / np.sqrt(var + eps), rtol=1e-13)
    # per channel: mean(y) = beta and var(y) = gamma^2 var/(var+eps)
    np.testing.assert_allclose(y.mean(axis=(0, 2, 3)), beta, atol=1e-12)
    np.testing.assert_allclose(y.var(axis=(0, 2, 3)), gamma ** 2 * var / (var + eps), rtol=1e-12)


def test_bn_constant_input_and_single_element():
    y, mean, invstd = oracle.bn_fwd(np.full((2, 2, 3, 3), 7.0), [2.0, 3.0], [0.5, -1.0], 1e-5)
    assert np.array_equal(y[:, 0], np.full((2, 3, 3), 0.5))
    assert np.array_equal(y[:, 1], np.full((2, 3, 3), -1.0))
    assert mean.tolist() == [7.0, 7.0]
    np.testing.assert_allclose(invstd, 1.0 / np.sqrt(1e-5), rtol=1e-14)
    y, _, _ = oracle.bn_fwd(np.array([[[[42.0]]]]), [3.0], [0.25], 1e-5)
    assert y.ravel().tolist() == [0.25]


def test_bn_affine_invariance():
    x = RNG.standard_normal((3, 2, 4, 4))
    g, b = [1.2, 0.8], [0.0, 1.0]
    y1, _, _ = oracle.bn_fwd(x, g, b, 0.0 + 1e-30)
    y2, _, _ = oracle.bn_fwd(5.0 * x - 11.0, g, b, 0.0 + 1e-30)
    np.testing.assert_allclose(y1, y2, rtol=1e-10, atol=1e-10)


def test_bn_against_torch():
    N, C, H, W = 3, 4, 6, 5
    x = RNG.standard_normal((N, C, H, W)) + 0.5
    gamma, beta = RNG.uniform(0.5, 1.5, C), RNG.standard_normal(C) * 0.1
    dy = RNG.standard_normal((N, C, H, W))
    xt = torch.from_numpy(x).requires_grad_(True)
    gt = torch.from_numpy(gamma).requires_grad_(True)
    bt = torch.from_numpy(beta).requires_grad_(True)
    yt = torch.nn.functional.batch_norm(xt, None, None, gt, bt, training=True, eps=1e-5)
    yt.backward(torch.from_numpy(dy))
    y, mean, invstd = oracle.bn_fwd(x, gamma, beta, 1e-5)
    np.testing.assert_allclose(y, yt.detach().numpy(), rtol=1e-11, atol=1e-11)
    dx, dgamma, dbeta = oracle.bn_bwd(x, dy, gamma, mean, invstd)
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(dgamma, gt.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dbeta, bt.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_bn_bwd_invariants_and_finite_differences():
    N, C, H, W = 2, 3, 4, 4
    x = RNG.standard_normal((N, C, H, W))
    gamma, beta = RNG.uniform(0.5, 1.5, C), RNG.standard_normal(C)
    dy = RNG.standard_normal((N, C, H, W))
    eps = 1e-5
    y, mean, invstd = oracle.bn_fwd(x, gamma, beta, eps)
    dx, dgamma, dbeta = oracle.bn_bwd(x, dy, gamma, mean, invstd)
    xhat = (x - mean.reshape(1, C, 1, 1)) * invstd.reshape(1, C, 1, 1)
    np.testing.assert_allclose(dx.sum(axis=(0, 2, 3)), 0.0, atol=1e-12)
    # sum(xhat^2) = M var/(var+eps), so sum(dx*xhat) = gamma*invstd*dgamma * eps*invstd^2
    # (exactly 0 only when eps = 0)
    np.testing.assert_allclose((dx * xhat).sum(axis=(0, 2, 3)), gamma * invstd * dgamma * eps * invstd ** 2,
                               rtol=1e-8, atol=1e-13)
    np.testing.assert_allclose(dbeta, dy.sum(axis=(0, 2, 3)), rtol=1e-13)

    def loss(xx, gg, bb):
        return float((oracle.bn_fwd(xx, gg, bb, eps)[0] * dy).sum())

    h = 1e-5
    for idx in [(0, 0, 0, 0), (1, 2, 3, 1), (0, 1, 2, 2)]:
        e = np.zeros_like(x)
        e[idx] = h
        fd = (loss(x + e, gamma, beta) - loss(x - e, gamma, beta)) / (2 * h)
        assert abs(fd - dx[idx]) <= 1e-6 * max(1.0, abs(fd))
    for c in range(C):
        e = np.zeros(C)
        e[c] = h
        fd = (loss(x, gamma + e, beta) - loss(x, gamma - e, beta)) / (2 * h)
        assert abs(fd - dgamma[c]) <= 1e-7 * max(1.0, abs(fd))
        fd = (loss(x, gamma, beta + e) - loss(x, gamma, beta - e)) / (2 * h)
        assert abs(fd - dbeta[c]) <= 1e-7 * max(1.0, abs(fd))


# ----------------------------------------------------------------- max-pool
def test_pool_hand_ties():
    x = np.zeros((1, 1, 4, 4))
    y, idx = oracle.maxpool_fwd(x, (2, 2), (2, 2))
    # all-equal windows: the top-left element of each window wins
    assert idx[0, 0].tolist() == [[0, 2], [8, 10]]
    x[0, 0, 0, 1] = x[0, 0, 1, 0] = 5.0      # two equal maxima: earlier row-major one
    x[0, 0, 3, 2] = x[0, 0, 3, 3] = 2.0
    y, idx = oracle.maxpool_fwd(x, (2, 2), (2, 2))
    assert idx[0, 0].tolist() == [[1, 2], [8, 14]]
    assert y[0, 0].tolist() == [[5.0, 0.0], [0.0, 2.0]]


def test_pool_padding_excluded():
    # all-negative input with padding: padded positions must never win
    x = -np.arange(1.0, 10.0).reshape(1, 1, 3, 3)
    y, idx = oracle.maxpool_fwd(x, (3, 3), (2, 2), (1, 1))
    assert y.shape == (1, 1, 2, 2)
    assert y[0, 0].tolist() == [[-1.0, -2.0], [-4.0, -5.0]]
    assert idx[0, 0].tolist() == [[0, 1], [3, 4]]


@pytest.mark.parametrize("geom", [((2, 2), (2, 2), (0, 0), 8, 8), ((3, 3), (2, 2), (0, 0), 13, 13),
                                  ((3, 3), (2, 2), (1, 1), 9, 12), ((3, 2), (1, 2), (1, 0), 7, 10)])
def test_pool_properties_and_torch(geom):
    kernel, stride, pad, H, W = geom
    x = np.round(RNG.standard_normal((2, 3, H, W)) * 2.0) / 2.0   # coarse grid: real ties
    x = np.maximum(x, 0.0)
    y, idx = oracle.maxpool_fwd(x, kernel, stride, pad)
    N, C, P, Q = y.shape
    flat = x.reshape(N, C, -1)
    assert np.array_equal(np.take_along_axis(flat, idx.reshape(N, C, -1).astype(np.int64), 2).reshape(y.shape), y)
    for p in range(P):
        for q in range(Q):
            h0, w0 = p * stride[0] - pad[0], q * stride[1] - pad[1]
            win = x[:, :, max(h0, 0):min(h0 + kernel[0], H), max(w0, 0):min(w0 + kernel[1], W)]
            assert np.array_equal(win.max(axis=(2, 3)), y[:, :, p, q])
            hh, ww = idx[:, :, p, q] // W, idx[:, :, p, q] % W
            assert ((hh >= max(h0, 0)) & (hh < h0 + kernel[0]) & (ww >= max(w0, 0)) & (ww < w0 + kernel[1])).all()
    yt, it = torch.nn.functional.max_pool2d(torch.from_numpy(x), kernel, stride, pad, return_indices=True)
    assert np.array_equal(y, yt.numpy())
    assert np.array_equal(idx, it.numpy().astype(np.int32))
    dy = RNG.standard_normal(y.shape)
    dx = oracle.maxpool_bwd(dy, idx, x.shape)
    np.testing.assert_allclose(dx.sum(), dy.sum(), rtol=1e-12)
    xt = torch.from_numpy(x).requires_grad_(True)
    torch.nn.functional.max_pool2d(xt, kernel, stride, pad).backward(torch.from_numpy(dy))
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-12, atol=1e-12)


def test_pool_bwd_overlap_sums():
    # 3x3 stride 1 windows over a single peak: every window picks the peak
    x = np.zeros((1, 1, 3, 3))
    x[0, 0, 1, 1] = 1.0
    y, idx = oracle.maxpool_fwd(x, (2, 2), (1, 1))
    assert (idx == 4).all()
    dx = oracle.maxpool_bwd(np.array([1.0, 2.0, 3.0, 4.0]).reshape(1, 1, 2, 2), idx, x.shape)
    assert dx[0, 0, 1, 1] == 10.0 and dx.sum() == 10.0


def test_pool_finite_differences_away_from_ties():
    x = RNG.permutation(36).astype(np.float64).reshape(1, 1, 6, 6)   # all distinct
    dy = RNG.standard_normal((1, 1, 2, 2))
    _, idx = oracle.maxpool_fwd(x, (3, 3), (3, 3))
    dx = oracle.maxpool_bwd(dy, idx, x.shape)

    def loss(xx):
        return float((oracle.maxpool_fwd(xx, (3, 3), (3, 3))[0] * dy).sum())

    for i in range(6):
        for j in range(6):
            e = np.zeros_like(x)
            e[0, 0, i, j] = 1e-3
            fd = (loss(x + e) - loss(x - e)) / 2e-3
            assert abs(fd - dx[0, 0, i, j]) < 1e-9


# ----------------------------------------------------------------- LRN
def test_lrn_hand_example():
    # one pixel, three channels 1, 2, 3; size 3, alpha 3 (so alpha / size = 1), beta 1, k 1:
    # s = 1 + (1 + 4), 1 + (1 + 4 + 9), 1 + (4 + 9) = 6, 15, 14
    x = np.array([1.0, 2.0, 3.0]).reshape(1, 3, 1, 1)
    y = oracle.lrn_fwd(x, size=3, alpha=3.0, beta=1.0, k=1.0).ravel()
    assert np.allclose(y, [1 / 6, 2 / 15, 3 / 14], rtol=1e-15, atol=0)
    # dy = (1, 0, 0): dx_0 = 1/6 - 2*1*1*(1*1/36) = 1/6 - 1/18, dx_1 = -2*2*(1/36), dx_2 = 0 (channel 0's window ends at 1)
    dx = oracle.lrn_bwd(x, np.array([1.0, 0.0, 0.0]).reshape(1, 3, 1, 1), size=3, alpha=3.0, beta=1.0, k=1.0).ravel()
    assert np.allclose(dx, [1 / 6 - 1 / 18, -4 / 36, 0.0], rtol=1e-14, atol=1e-16)


def test_lrn_special_cases():
    x = RNG.standard_normal((2, 7, 3, 4))
    dy = RNG.standard_normal(x.shape)
    # a window of one channel: elementwise
    y = oracle.lrn_fwd(x, size=1, alpha=0.3, beta=0.75, k=2.0)
    assert np.allclose(y, x / (2.0 + 0.3 * x * x) ** 0.75, rtol=1e-14)
    # alpha = 0: a constant factor both ways
    assert np.allclose(oracle.lrn_fwd(x, 5, 0.0, 0.75, 2.0), x * 2.0 ** -0.75, rtol=1e-15)
    assert np.allclose(oracle.lrn_bwd(x, dy, 5, 0.0, 0.75, 2.0), dy * 2.0 ** -0.75, rtol=1e-15)
    # all channels equal to v: the window of channel c holds min(c, h) + min(C-1-c, h) + 1 channels
    C, size, v = 9, 5, 1.5
    xc = np.full((1, C, 2, 2), v)
    cnt = np.array([min(c, 2) + min(C - 1 - c, 2) + 1 for c in range(C)], dtype=np.float64)
    want = v / (1.0 + 0.5 / size * cnt * v * v) ** 0.75
    assert np.allclose(oracle.lrn_fwd(xc, size, 0.5, 0.75, 1.0)[0, :, 1, 1], want, rtol=1e-14)


def test_lrn_matches_torch_and_finite_differences():
    x = RNG.standard_normal((2, 11, 3, 5)) * 2.0
    dy = RNG.standard_normal(x.shape)
    for size, alpha, beta, k in ((5, 1e-1, 0.75, 2.0), (3, 0.7, 0.5, 1.0), (7, 2.0, 1.25, 0.5)):
        xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
        yt = torch.nn.functional.local_response_norm(xt, size, alpha=alpha, beta=beta, k=k)
        yt.backward(torch.tensor(dy))
        assert np.allclose(oracle.lrn_fwd(x, size, alpha, beta, k), yt.detach().numpy(), rtol=1e-12, atol=1e-14)
        dx = oracle.lrn_bwd(x, dy, size, alpha, beta, k)
        assert np.allclose(dx, xt.grad.numpy(), rtol=1e-11, atol=1e-13)
        # central differences of sum(dy * y) in a few coordinates
        f = lambda z: float((dy * oracle.lrn_fwd(z, size, alpha, beta, k)).sum())
        for idx in [(0, 0, 0, 0), (1, 5, 2, 3), (0, 10, 1, 4), (1, 1, 0, 2)]:
            h = 1e-6
            xp, xm = x.copy(), x.copy()
            xp[idx] += h
            xm[idx] -= h
            assert abs((f(xp) - f(xm)) / (2 * h) - dx[idx]) <= 1e-7 * max(1.0, abs(dx[idx]))
