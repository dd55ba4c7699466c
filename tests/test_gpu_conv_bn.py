"""GPU parity of the CONV forward that also takes the batch statistics of its output, and of the
BN passes that start from given statistics.

Bars: y bit-identical to sn_conv2d_fwd with the same algorithm and workspace; mean and invstd
within 1e-5 (relative L2) of the oracle's statistics of that stored y; the normalisation passes
bit-identical to the calls that take the statistics themselves.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_1801_04380_amd as sn
from paper_1801_04380_amd import workloads as wl
from _parity import DT, f64, rel_l2, shape_of, workspace
from test_gpu_conv import _algos

pytestmark = pytest.mark.gpu

L = wl._L
# every kernel family that takes the statistics from its accumulators (3x3 with the packed filter in
# its tilings, 64-channel tiles, 1x1, other filters, zero-workspace), and shapes that fall back to a
# pass over y (strides, fp32, the explicit algorithm)
CASES = [
    (L("wide", 32, 24, 40, 160, 3, 3, (1, 1), (1, 1)), 3),
    (L("w28", 64, 28, 28, 128, 3, 3, (1, 1), (1, 1)), 3),
    (L("w14_split", 64, 14, 14, 128, 3, 3, (1, 1), (1, 1)), 4),
    (L("k64", 48, 20, 36, 64, 3, 3, (1, 1), (1, 1)), 3),
    (L("k48_w72", 104, 12, 72, 48, 3, 3, (1, 1), (1, 1)), 3),
    (L("rf_c64_k64", 64, 20, 40, 64, 3, 3, (1, 1), (1, 1)), 3),
    (L("rf_c32_k40_pad0", 32, 12, 72, 40, 3, 3, (1, 1), (0, 0)), 2),
    (L("first3", 3, 40, 40, 64, 3, 3, (1, 1), (1, 1), relu_in=False), 2),
    (L("few_c3_w150", 3, 9, 150, 70, 3, 3, (1, 1), (1, 1), relu_in=False), 2),
    (L("few_c3_s2_valid", 3, 37, 41, 32, 3, 3, (2, 2), (0, 0), relu_in=False), 3),
    (L("ragged3x3", 19, 37, 29, 70, 3, 3, (1, 1), (1, 1)), 3),
    (L("1x1", 96, 14, 14, 160, 1, 1), 3),
    (L("5x5", 24, 27, 27, 32, 5, 5, (1, 1), (2, 2)), 2),
    (L("s2_3x3", 16, 33, 33, 40, 3, 3, (2, 2), (1, 1)), 2),
    (L("one_pixel_out", 5, 3, 3, 7, 3, 3), 1),
]


@pytest.mark.parametrize("dtype,out", [("bf16", "bf16"), ("bf16", "f32"), ("f32", "f32")])
@pytest.mark.parametrize("case", CASES, ids=[c[0].name for c in CASES])
def test_conv_fwd_bn_stats(case, dtype, out):
    layer, N = case
    x, w, _ = wl.conv_inputs(layer, N, dtype, seed=7)
    # a mean away from 0 in some channels: shift the filter's taps of every third output channel
    w = w.float()
    w[::3] += 0.05
    w = w.to(DT[dtype])
    shape = shape_of(layer, N, dtype, out)
    P, Q = sn.sn_out_dim(layer.H, layer.pad[0], layer.R, layer.stride[0]), sn.sn_out_dim(layer.W, layer.pad[1], layer.S, layer.stride[1])
    xd, wd = x.cuda(), w.cuda()
    scratch = torch.empty(max(sn.sn_conv_bn_stats_scratch_bytes(shape), 16), dtype=torch.uint8, device="cuda")
    eps = 1e-5
    for algo, ws_bytes in _algos(shape, sn.SN_CONV_FWD):
        print("case", layer.name, dtype, "->", out, "algo", sn.ALGO_NAMES[algo], "ws", ws_bytes, flush=True)
        ws = workspace(ws_bytes)
        y_ref = torch.full((N, layer.K, P, Q), float("nan"), dtype=DT[out], device="cuda")
        sn.sn_conv2d_fwd(xd, wd, y_ref, shape, algo, ws)
        y = torch.full_like(y_ref, float("nan"))
        mean = torch.full((layer.K,), float("nan"), device="cuda")
        invstd = torch.full((layer.K,), float("nan"), device="cuda")
        scratch.fill_(0xff)
        sn.sn_conv2d_fwd_bn_stats(xd, wd, y, shape, mean, invstd, scratch, algo, ws, eps)
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref)
        _, mo, io = oracle.bn_fwd(f64(y), np.ones(layer.K), np.zeros(layer.K), eps)
        assert rel_l2(f64(mean), mo) <= 1e-5
        assert rel_l2(f64(invstd), io) <= 1e-5
        # a replay gives the same bits
        mean2, invstd2 = torch.empty_like(mean), torch.empty_like(invstd)
        sn.sn_conv2d_fwd_bn_stats(xd, wd, y, shape, mean2, invstd2, scratch, algo, ws, eps)
        torch.cuda.synchronize()
        assert torch.equal(mean, mean2) and torch.equal(invstd, invstd2)


def test_conv_fwd_bn_stats_scratch_too_small():
    layer, N = CASES[0]
    shape = shape_of(layer, N, "bf16", "bf16")
    x, w, _ = wl.conv_inputs(layer, N, "bf16", seed=7)
    y = torch.empty((N, layer.K, layer.H, layer.W), dtype=torch.bfloat16, device="cuda")
    m, i = torch.empty(layer.K, device="cuda"), torch.empty(layer.K, device="cuda")
    need = sn.sn_conv_bn_stats_scratch_bytes(shape)
    assert need > 0 and need % 256 == 0
    small = torch.empty(need - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(sn.SnError) as e:
        sn.sn_conv2d_fwd_bn_stats(x.cuda(), w.cuda(), y, shape, m, i, small)
    assert e.value.status == 3   # SN_ERR_WORKSPACE_TOO_SMALL


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(4, 16, 16, 16), (40, 4, 64, 64), (3, 5, 7, 9), (2, 3, 1, 1), (36, 2, 56, 56)],
                         ids=lambda s: "x".join(map(str, s)))
def test_bn_apply_from_given_statistics(shape, dtype):
    N, C, H, W = shape
    x = (wl.activation(shape, "f32", 5) * 1.5 + 0.7).to(DT[dtype]).cuda()
    gamma, beta = (t.cuda() for t in wl.bn_params(C, 5))
    new = lambda: torch.empty(C, device="cuda")
    y, mean, invstd = torch.empty_like(x), new(), new()
    sn.sn_bn_fwd(x, gamma, beta, y, mean, invstd)
    a, m2, i2 = torch.empty_like(x), new(), new()
    sn.sn_bn_relu_fwd(x, gamma, beta, a, m2, i2)
    y_ap = torch.full_like(x, float("nan"))
    a_ap = torch.full_like(x, float("nan"))
    sn.sn_bn_apply(x, gamma, beta, mean, invstd, y_ap, relu=False)
    sn.sn_bn_apply(x, gamma, beta, mean, invstd, a_ap, relu=True)
    torch.cuda.synchronize()
    assert torch.equal(y_ap, y) and torch.equal(a_ap, a)
    if H % 2 == 0 and W % (4 if dtype == "bf16" else 2) == 0:
        pooled = torch.empty((N, C, H // 2, W // 2), dtype=DT[dtype], device="cuda")
        idx = torch.empty((N, C, H // 2, W // 2), dtype=torch.int32, device="cuda")
        sn.sn_bn_relu_pool2_fwd(x, gamma, beta, pooled, idx, m2, i2)
        p_ap, i_ap = torch.full_like(pooled, float("nan")), torch.full_like(idx, -7)
        sn.sn_bn_relu_pool2_apply(x, gamma, beta, mean, invstd, p_ap, i_ap)
        torch.cuda.synchronize()
        assert torch.equal(p_ap, pooled) and torch.equal(i_ap, idx)
