"""GPU parity of the cheap layers (ReLU, BN, LRN, max-pool) against the fp64 oracle.

Bars: pool indices bit-exact; values relative L2 <= 1e-5 (fp32 storage) or
<= 5e-3 (bf16 storage, oracle fed the bf16-rounded inputs).  ReLU and pool
forward only move values, so they must match exactly in either storage type.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_1801_04380_amd as sn
from paper_1801_04380_amd import workloads as wl
from _parity import DT, TOL, f64, rel_l2

pytestmark = pytest.mark.gpu

# sizes: a ragged tail below one vector, several workgroups, odd plane sizes
FLAT_SIZES = [0, 1, 7, 8, 9, 1023, 4096, 100003, 5 * 1024 * 1024 + 13]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", FLAT_SIZES)
def test_relu(n, dtype):
    x = wl.activation((n,), dtype, seed=n + 1)
    dy = wl.activation((n,), dtype, seed=n + 2)
    if n >= 9:
        x[3] = 0.0
        x[5] = -0.0
    xd, dyd = x.cuda(), dy.cuda()
    y = torch.full_like(xd, float("nan"))
    dx = torch.full_like(xd, float("nan"))
    sn.sn_relu_fwd(xd, y)
    sn.sn_relu_bwd(xd, dyd, dx)
    dx2 = torch.full_like(xd, float("nan"))
    sn.sn_relu_bwd(y, dyd, dx2)              # gating on the output is the same gate
    torch.cuda.synchronize()
    assert np.array_equal(f64(y), oracle.relu_fwd(f64(x)))
    want = oracle.relu_bwd(f64(x), f64(dy))
    assert np.array_equal(f64(dx), want)
    assert np.array_equal(f64(dx2), want)
    if n:
        z = xd.clone()
        sn.sn_relu_fwd(z, z)                 # in place
        torch.cuda.synchronize()
        assert torch.equal(z, y)


BN_SHAPES = [(2, 3, 5, 7), (4, 16, 14, 14), (3, 8, 7, 7), (2, 5, 35, 35), (8, 64, 56, 56), (2, 4, 224, 224),
             (1, 1, 1, 1), (1, 3, 1, 1), (2, 2, 1, 1), (1, 2, 1, 3), (64, 32, 7, 7), (2, 130, 9, 9),
             # a channel that just fits the one-pass kernels' registers, one just past that, 8-byte vectors
             (32, 6, 56, 56), (34, 3, 56, 56), (32, 8, 14, 14),
             # long channels with many planes: whole slices and a ragged last one
             (16, 64, 64, 64), (12, 130, 36, 40),
             # planes that are no whole number of 8-byte vectors (16-byte vectors at any alignment, the last one of
             # a plane moved back): 30 and 9 pixels, channels for the 256- and the 1024-thread build, the longest that takes this path and one past it
             (3, 4, 5, 6), (5, 3, 3, 3), (64, 4, 17, 17), (26, 8, 35, 35), (27, 2, 35, 35)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", BN_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_bn(shape, dtype):
    N, C, H, W = shape
    seed = N * 1000 + C * 10 + H
    # a mean well away from 0 and a different scale per channel
    x = wl.activation(shape, "f32", seed, scale=1.0)
    x = (x * torch.linspace(0.5, 3.0, C).view(1, C, 1, 1) + torch.linspace(-2.0, 5.0, C).view(1, C, 1, 1))
    x = x.to(DT[dtype])
    dy = wl.activation(shape, dtype, seed + 1)
    gamma, beta = wl.bn_params(C, seed)
    eps = 1e-5
    xd, dyd, gd, bd = x.cuda(), dy.cuda(), gamma.cuda(), beta.cuda()
    y = torch.full_like(xd, float("nan"))
    mean = torch.empty(C, device="cuda")
    invstd = torch.empty(C, device="cuda")
    sn.sn_bn_fwd(xd, gd, bd, y, mean, invstd, eps)
    dx = torch.full_like(xd, float("nan"))
    dgamma = torch.empty(C, device="cuda")
    dbeta = torch.empty(C, device="cuda")
    sn.sn_bn_bwd(xd, dyd, gd, mean, invstd, dx, dgamma, dbeta)
    # a replay must reproduce the first run bit for bit
    y2 = torch.empty_like(y)
    mean2, invstd2 = torch.empty_like(mean), torch.empty_like(invstd)
    sn.sn_bn_fwd(xd, gd, bd, y2, mean2, invstd2, eps)
    torch.cuda.synchronize()
    assert torch.equal(y, y2) and torch.equal(mean, mean2) and torch.equal(invstd, invstd2)

    # BN + ReLU in one pass: the same statistics, and exactly the ReLU of the BN output
    a = torch.full_like(xd, float("nan"))
    mean3, invstd3 = torch.empty_like(mean), torch.empty_like(invstd)
    sn.sn_bn_relu_fwd(xd, gd, bd, a, mean3, invstd3, eps)
    a_ref = torch.empty_like(y)
    sn.sn_relu_fwd(y, a_ref)
    torch.cuda.synchronize()
    assert torch.equal(mean, mean3) and torch.equal(invstd, invstd3)
    assert torch.equal(a, a_ref)

    yo, mo, io = oracle.bn_fwd(f64(x), f64(gamma), f64(beta), eps)
    tol = TOL[dtype]
    assert rel_l2(f64(a), oracle.relu_fwd(yo)) <= tol
    assert rel_l2(f64(mean), mo) <= 1e-5
    assert rel_l2(f64(invstd), io) <= 1e-5
    assert rel_l2(f64(y), yo) <= tol
    # ReLU backward + BN backward in one call: exactly the two calls in a row
    g = torch.empty_like(dyd)
    sn.sn_relu_bwd(a, dyd, g)
    dx_ref = torch.full_like(xd, float("nan"))
    dg_ref, db_ref = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
    sn.sn_bn_bwd(xd, g, gd, mean, invstd, dx_ref, dg_ref, db_ref)
    dx_f = torch.full_like(xd, float("nan"))
    dg_f, db_f = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
    sn.sn_bn_relu_bwd(xd, dyd, gd, bd, mean, invstd, dx_f, dg_f, db_f)
    torch.cuda.synchronize()
    assert torch.equal(dx_f, dx_ref) and torch.equal(dg_f, dg_ref) and torch.equal(db_f, db_ref)
    go = oracle.relu_bwd(f64(a), f64(dy))
    dxo2, dgo2, dbo2 = oracle.bn_bwd(f64(x), go, f64(gamma), f64(mean), f64(invstd))
    assert rel_l2(f64(dg_f), dgo2) <= 1e-5 and rel_l2(f64(db_f), dbo2) <= 1e-5
    if N * H * W > 4:
        assert rel_l2(f64(dx_f), dxo2) <= tol

    # backward from the statistics the GPU saved (what the API consumes)
    dxo, dgo, dbo = oracle.bn_bwd(f64(x), f64(dy), f64(gamma), f64(mean), f64(invstd))
    assert rel_l2(f64(dgamma), dgo) <= 1e-5
    assert rel_l2(f64(dbeta), dbo) <= 1e-5
    if N * H * W > 4:
        assert rel_l2(f64(dx), dxo) <= tol
    else:
        # with a handful of elements per channel dx is a difference of nearly equal terms
        # (exactly 0 for M = 1), so the error is measured against the size of those terms
        terms = f64(gamma).reshape(1, C, 1, 1) * f64(invstd).reshape(1, C, 1, 1) * f64(dy)
        assert np.linalg.norm(f64(dx) - dxo) <= tol * np.linalg.norm(terms)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,H", [(4, 16), (40, 64)], ids=["one_pass", "two_pass"])
def test_bn_relu_bwd_gate_edges(N, H, dtype):
    """The pair's backward re-derives the ReLU gate from x.  Where the BN output is 0, negative,
    or so small that its stored value rounds to 0, it must decide as a read of the stored output does."""
    C, W = 6, H
    x = wl.activation((N, C, H, W), dtype, 77).cuda()
    x[:, 1] = 0.25                                    # a constant channel: BN output exactly beta
    dy = wl.activation((N, C, H, W), dtype, 78).cuda()
    # channel 0: outputs around the smallest bf16 subnormal (2^-133); 1: exactly 0; 2: all negative;
    # 3: tiny negative gamma; 4, 5: ordinary
    gamma = torch.tensor([2.0 ** -133, 1.0, 1e-3, -(2.0 ** -134), 1.0, -0.7], device="cuda")
    beta = torch.tensor([0.0, 0.0, -1.0, 2.0 ** -135, 0.1, 0.2], device="cuda")
    mean, invstd = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
    a = torch.empty_like(x)
    sn.sn_bn_relu_fwd(x, gamma, beta, a, mean, invstd, 1e-5)
    g = torch.empty_like(dy)
    sn.sn_relu_bwd(a, dy, g)
    dx_ref, dx_f = torch.empty_like(x), torch.empty_like(x)
    dg_ref, db_ref = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
    dg_f, db_f = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
    sn.sn_bn_bwd(x, g, gamma, mean, invstd, dx_ref, dg_ref, db_ref)
    sn.sn_bn_relu_bwd(x, dy, gamma, beta, mean, invstd, dx_f, dg_f, db_f)
    torch.cuda.synchronize()
    assert torch.equal(db_f, db_ref) and torch.equal(dg_f, dg_ref) and torch.equal(dx_f, dx_ref)
    assert float(db_ref[1]) == 0.0 and float(db_ref[2]) == 0.0     # nothing passes where the output is <= 0
    assert float(db_ref[4]) != 0.0


# one-pass statistics with 16- and 8-byte row accesses, the three-kernel path with both, a single
# window per plane, rows of one access, a wide plane
POOL2_PAIR_SHAPES = [(4, 16, 16, 16), (2, 5, 4, 12), (40, 4, 64, 64), (40, 3, 56, 60), (3, 7, 2, 4),
                     (2, 3, 6, 8), (32, 6, 56, 56), (2, 2, 2, 304), (36, 2, 56, 56),
                     (16, 64, 64, 64), (12, 130, 36, 40)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", POOL2_PAIR_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_bn_relu_pool2(shape, dtype):
    """BN + ReLU + 2x2 pool in one call, forward and backward: bit-identical to the separate calls
    (themselves checked against the oracle above), and the chain against the oracle's."""
    N, C, H, W = shape
    seed = N * 1000 + C * 10 + H
    x = wl.activation(shape, "f32", seed, scale=1.0)
    x = (x * torch.linspace(0.5, 3.0, C).view(1, C, 1, 1) + torch.linspace(-2.0, 5.0, C).view(1, C, 1, 1))
    x = (torch.round(x * 8.0) / 8.0).to(DT[dtype])          # coarse values: equal maxima inside windows
    gamma, beta = wl.bn_params(C, seed)
    dp = wl.activation((N, C, H // 2, W // 2), dtype, seed + 1)
    xd, gd, bd, dpd = x.cuda(), gamma.cuda(), beta.cuda(), dp.cuda()
    new = lambda *s, dt=torch.float32: torch.empty(*s, dtype=dt, device="cuda")

    # the separate calls
    a, mean, invstd = torch.empty_like(xd), new(C), new(C)
    sn.sn_bn_relu_fwd(xd, gd, bd, a, mean, invstd)
    pooled_ref = torch.empty_like(dpd)
    idx_ref = new(N, C, H // 2, W // 2, dt=torch.int32)
    sn.sn_maxpool_fwd(a, pooled_ref, idx_ref, (2, 2), (2, 2))
    g = torch.empty_like(xd)
    sn.sn_maxpool_bwd(dpd, idx_ref, g, (2, 2), (2, 2))
    dx_ref, dg_ref, db_ref = torch.empty_like(xd), new(C), new(C)
    sn.sn_bn_relu_bwd(xd, g, gd, bd, mean, invstd, dx_ref, dg_ref, db_ref)

    # the single calls
    pooled = torch.full_like(dpd, float("nan"))
    idx = torch.full((N, C, H // 2, W // 2), -7, dtype=torch.int32, device="cuda")
    mean2, invstd2 = new(C), new(C)
    sn.sn_bn_relu_pool2_fwd(xd, gd, bd, pooled, idx, mean2, invstd2)
    dx, dg, db = torch.full_like(xd, float("nan")), new(C), new(C)
    sn.sn_bn_relu_pool2_bwd(xd, dpd, idx, gd, bd, mean2, invstd2, dx, dg, db)
    torch.cuda.synchronize()
    assert torch.equal(mean2, mean) and torch.equal(invstd2, invstd)
    assert torch.equal(idx, idx_ref) and torch.equal(pooled, pooled_ref)
    assert torch.equal(db, db_ref) and torch.equal(dg, dg_ref) and torch.equal(dx, dx_ref)

    # the chain against the oracle: pooling and routing by the GPU's (checked) indices are exact on
    # the stored activations, the BN arithmetic is within the storage type's tolerance
    tol = TOL[dtype]
    yo, _, _ = oracle.bn_fwd(f64(x), f64(gamma), f64(beta), 1e-5)
    ao = oracle.relu_fwd(yo)
    po, _ = oracle.maxpool_fwd(ao, (2, 2), (2, 2))
    assert rel_l2(f64(pooled), po) <= tol
    a_st, io = oracle.maxpool_fwd(f64(a), (2, 2), (2, 2))
    assert np.array_equal(idx.cpu().numpy(), io) and np.array_equal(f64(pooled), a_st)
    go = oracle.relu_bwd(f64(a), oracle.maxpool_bwd(f64(dp), io, shape))
    dxo, dgo, dbo = oracle.bn_bwd(f64(x), go, f64(gamma), f64(mean), f64(invstd))
    assert rel_l2(f64(dg), dgo) <= 1e-5 and rel_l2(f64(db), dbo) <= 1e-5
    assert rel_l2(f64(dx), dxo) <= tol


def test_bn_relu_pool2_unsupported():
    """Shapes the single call does not take are refused, not mishandled."""
    x = torch.zeros(2, 2, 14, 14, dtype=torch.bfloat16, device="cuda")     # rows of 14 bf16: no 8-byte access
    one = torch.zeros(2, device="cuda")
    pooled = torch.zeros(2, 2, 7, 7, dtype=torch.bfloat16, device="cuda")
    idx = torch.zeros(2, 2, 7, 7, dtype=torch.int32, device="cuda")
    with pytest.raises(sn.SnError) as e:
        sn.sn_bn_relu_pool2_fwd(x, one, one, pooled, idx, one.clone(), one.clone())
    assert e.value.status == 2   # SN_ERR_UNSUPPORTED
    x = torch.zeros(2, 2, 5, 8, dtype=torch.bfloat16, device="cuda")       # odd height
    with pytest.raises(sn.SnError) as e:
        sn.sn_bn_relu_pool2_fwd(x, one, one, pooled, idx, one.clone(), one.clone())
    assert e.value.status == 2   # SN_ERR_UNSUPPORTED


LRN_SHAPES = [(2, 16, 8, 8), (2, 96, 27, 27), (1, 3, 5, 7), (3, 2, 4, 4), (2, 1, 3, 3), (2, 256, 13, 13),
              (4, 40, 16, 20), (2, 6, 5, 6), (3, 4, 1, 1), (1, 7, 55, 55)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("params", [(5, 1e-4, 0.75, 2.0), (3, 1.0, 0.5, 1.0), (9, 2.0, 1.25, 0.5), (1, 0.3, 0.75, 2.0),
                                    (7, 0.0, 0.75, 2.0)], ids=lambda p: "n%d_a%g" % (p[0], p[1]))
@pytest.mark.parametrize("shape", LRN_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_lrn(shape, params, dtype):
    size, alpha, beta, k = params
    seed = shape[1] * 100 + shape[2] + size
    x = wl.activation(shape, dtype, seed, scale=2.0)
    dy = wl.activation(shape, dtype, seed + 1)
    xd, dyd = x.cuda(), dy.cuda()
    y = torch.full_like(xd, float("nan"))
    dx = torch.full_like(xd, float("nan"))
    sn.sn_lrn_fwd(xd, y, size, alpha, beta, k)
    sn.sn_lrn_bwd(xd, dyd, dx, size, alpha, beta, k)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert rel_l2(f64(y), oracle.lrn_fwd(f64(x), size, alpha, beta, k)) <= tol
    assert rel_l2(f64(dx), oracle.lrn_bwd(f64(x), f64(dy), size, alpha, beta, k)) <= tol


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("params", [(5, 1e-4, 0.75, 2.0), (3, 1.0, 0.5, 1.0), (9, 2.0, 1.25, 0.5)],
                         ids=lambda p: "n%d_a%g" % (p[0], p[1]))
@pytest.mark.parametrize("shape", LRN_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_relu_lrn_one_pass(shape, params, dtype):
    """ReLU + LRN in one call each way: the oracle's ReLU and LRN composed, and bit for bit the two separate calls."""
    size, alpha, beta, k = params
    seed = shape[1] * 100 + shape[2] + size + 7
    x = wl.activation(shape, dtype, seed, scale=2.0)
    dy = wl.activation(shape, dtype, seed + 1)
    xd, dyd = x.cuda(), dy.cuda()
    y = torch.full_like(xd, float("nan"))
    dx = torch.full_like(xd, float("nan"))
    sn.sn_relu_lrn_fwd(xd, y, size, alpha, beta, k)
    sn.sn_relu_lrn_bwd(xd, dyd, dx, size, alpha, beta, k)
    a, y2, g, dx2 = (torch.full_like(xd, float("nan")) for _ in range(4))
    sn.sn_relu_fwd(xd, a)
    sn.sn_lrn_fwd(a, y2, size, alpha, beta, k)
    sn.sn_lrn_bwd(a, dyd, g, size, alpha, beta, k)
    sn.sn_relu_bwd(xd, g, dx2)
    torch.cuda.synchronize()
    assert torch.equal(y, y2) and torch.equal(dx, dx2)
    tol = TOL[dtype]
    ao = oracle.relu_fwd(f64(x))
    assert rel_l2(f64(y), oracle.lrn_fwd(ao, size, alpha, beta, k)) <= tol
    assert rel_l2(f64(dx), oracle.relu_bwd(f64(x), oracle.lrn_bwd(ao, f64(dy), size, alpha, beta, k))) <= tol


POOL_CASES = [((2, 16, 16, 16), (2, 2), (2, 2), (0, 0)), ((2, 8, 55, 55), (3, 3), (2, 2), (0, 0)),
              ((3, 5, 13, 13), (3, 3), (2, 2), (0, 0)), ((2, 6, 35, 35), (3, 3), (2, 2), (0, 0)),
              ((2, 4, 17, 17), (3, 3), (2, 2), (0, 0)), ((1, 3, 9, 12), (3, 3), (2, 2), (1, 1)),
              ((2, 3, 7, 10), (3, 2), (1, 2), (1, 0)), ((1, 1, 1, 1), (1, 1), (1, 1), (0, 0)),
              ((2, 4, 224, 224), (2, 2), (2, 2), (0, 0)), ((2, 3, 15, 15), (2, 2), (2, 2), (0, 0)),
              ((1, 2, 8, 8), (3, 3), (1, 1), (1, 1)), ((3, 5, 14, 14), (2, 2), (2, 2), (0, 0)),
              ((1, 2, 2, 2), (2, 2), (2, 2), (0, 0)), ((2, 3, 33, 20), (2, 2), (2, 2), (0, 0)),
              ((1, 2, 6, 300), (2, 2), (2, 2), (0, 0)),
              # 3x3 / stride 2 backward by row pieces of 8 columns: wide rows, padding, a column no window covers
              ((1, 2, 10, 150), (3, 3), (2, 2), (0, 0)), ((2, 3, 12, 40), (3, 3), (2, 2), (1, 1)),
              ((1, 2, 8, 8), (3, 3), (2, 2), (0, 0)), ((1, 2, 4, 3), (3, 3), (2, 2), (1, 1))]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", POOL_CASES, ids=lambda c: "x".join(map(str, c[0])) + "_k%d%d_s%d%d_p%d%d" % (c[1] + c[2] + c[3]))
def test_maxpool(case, dtype):
    shape, kernel, stride, pad = case
    N, C, H, W = shape
    # after a ReLU, coarsely quantised: all-zero windows and equal maxima are common
    x = wl.activation(shape, "f32", seed=H * 31 + W, relu=True)
    x = (torch.round(x * 4.0) / 4.0).to(DT[dtype])
    yo, io = oracle.maxpool_fwd(f64(x), kernel, stride, pad)
    P, Q = yo.shape[2:]
    dy = wl.activation((N, C, P, Q), dtype, seed=H * 31 + W + 1)
    xd, dyd = x.cuda(), dy.cuda()
    y = torch.full((N, C, P, Q), float("nan"), dtype=DT[dtype], device="cuda")
    idx = torch.full((N, C, P, Q), -7, dtype=torch.int32, device="cuda")
    sn.sn_maxpool_fwd(xd, y, idx, kernel, stride, pad)
    dx = torch.full_like(xd, float("nan"))
    sn.sn_maxpool_bwd(dyd, idx, dx, kernel, stride, pad)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), io)           # bit-exact, ties included
    assert np.array_equal(f64(y), yo)
    dxo = oracle.maxpool_bwd(f64(dy), io, shape)
    if kernel[0] <= stride[0] and kernel[1] <= stride[1]:
        assert np.array_equal(f64(dx), dxo)                # no overlap: pure routing
    else:
        assert rel_l2(f64(dx), dxo) <= TOL[dtype]


def test_measured_ceilings_are_sane():
    """sn_measure_ceiling: every kind runs, stays below the datasheet peak it is quoted beside, and the
    operand-fed MFMA loop does not beat the register-resident one; bad arguments are refused."""
    buf = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
    bf16 = sn.sn_measure_ceiling(sn.SN_CEIL_MFMA_BF16, buf, iters=2)
    fed = sn.sn_measure_ceiling(sn.SN_CEIL_MFMA_BF16_FED, buf, iters=2)
    f32 = sn.sn_measure_ceiling(sn.SN_CEIL_MFMA_F32, buf, iters=2)
    assert 500.0 < bf16 <= 2600.0 and 10.0 < f32 <= 165.0
    assert 300.0 < fed <= bf16 * 1.02
    for kind in (sn.SN_CEIL_COPY, sn.SN_CEIL_READ, sn.SN_CEIL_WRITE):
        assert 1000.0 < sn.sn_measure_ceiling(kind, buf, iters=2) <= 8000.0
    with pytest.raises(sn.SnError):
        sn.sn_measure_ceiling(6, buf)                                   # no such kind
    with pytest.raises(sn.SnError):
        sn.sn_measure_ceiling(sn.SN_CEIL_MFMA_BF16_FED, buf[: 2 << 20])    # needs the source and the sink
