"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times (autotuned plan under the configuration's largest
workspace budget, SN_ALGO_AUTO).  The fp64 oracle cannot produce whole outputs at
these sizes in seconds, so it computes sampled output elements one by one
(conv2d_*_at): corners, edges and seeded random positions.  The cheap layers are
checked in full on the largest activation of the VGG-shaped configuration.

Bars as in the small-size tests: relative L2 <= 5e-3 over the sample for bf16
inputs; ReLU and pool values exact, pool indices bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_1801_04380_amd as sn
from paper_1801_04380_amd import workloads as wl
from _parity import f64, rel_l2, shape_of

pytestmark = pytest.mark.gpu

# (configuration, layer name)
LAYERS = [(3, "conv1_1"), (3, "conv1_2"), (3, "conv2_1"), (3, "conv3_2"), (3, "conv4_2"), (3, "conv5_3"),
          (2, "conv2"), (2, "conv4"), (4, "s2_project"), (4, "s3_conv3x3"), (4, "s3_conv3x3_s2"),
          (5, "b_1x7"), (5, "b_7x1"), (5, "a_5x5_48_64")]
NSAMPLE = 40


def _positions(dims, rng):
    """Corners, a few edge points and seeded random positions of an index space."""
    pts = set()
    for mask in range(1 << len(dims)):
        pts.add(tuple((d - 1) if (mask >> i) & 1 else 0 for i, d in enumerate(dims)))
    while len(pts) < NSAMPLE + (1 << len(dims)):
        pts.add(tuple(int(rng.integers(0, d)) for d in dims))
    return sorted(pts)


@pytest.mark.parametrize("cfg_no,name", LAYERS, ids=["cfg%d-%s" % c for c in LAYERS])
def test_conv_full_size_sampled(cfg_no, name):
    cfg = wl.CONFIGS[cfg_no]
    N, dtype = cfg["N"], cfg["dtype"]
    li, layer = [(i, l) for i, l in enumerate(cfg["layers"]) if l.name == name][0]
    x, w, dy = wl.conv_inputs(layer, N, dtype, wl.layer_seed(cfg_no, li))
    P, Q = wl.out_hw(layer)
    shape = shape_of(layer, N, dtype, dtype)
    budget = max(b for b in cfg["budgets"] if b is not None)
    ws = torch.empty(max(budget, 256), dtype=torch.uint8, device="cuda") if budget else None
    xd, wd, dyd = x.cuda(), w.cuda(), dy.cuda()
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    y = torch.full((N, layer.K, P, Q), float("nan"), dtype=tdt, device="cuda")
    dx = torch.full_like(xd, float("nan"))
    dw = torch.full(tuple(w.shape), float("nan"), dtype=torch.float32, device="cuda")
    calls = {sn.SN_CONV_FWD: (sn.sn_conv2d_fwd, xd, wd, y), sn.SN_CONV_BWD_DATA: (sn.sn_conv2d_bwd_data, dyd, wd, dx),
             sn.SN_CONV_BWD_FILTER: (sn.sn_conv2d_bwd_filter, xd, dyd, dw)}
    for d, (fn, a, b, out) in calls.items():
        sn.sn_conv_autotune(d, a, b, out, shape, ws, iters=1)
        out.fill_(float("nan"))
        fn(a, b, out, shape, sn.SN_ALGO_AUTO, ws)
    torch.cuda.synchronize()
    assert not torch.isnan(y).any() and not torch.isnan(dx).any() and not torch.isnan(dw).any()
    rng = np.random.default_rng(cfg_no * 100 + li)
    xo, wo, dyo = f64(x), f64(w), f64(dy)
    yc, dxc, dwc = y.cpu(), dx.cpu(), dw.cpu()
    got, ref = [], []
    for (n, k, p, q) in _positions((N, layer.K, P, Q), rng):
        got.append(float(yc[n, k, p, q]))
        ref.append(oracle.conv2d_fwd_at(xo, wo, layer.stride, layer.pad, n, k, p, q))
    assert rel_l2(got, ref) <= 5e-3, ("fwd", name, rel_l2(got, ref))
    got, ref = [], []
    for (n, c, h, v) in _positions((N, layer.C, layer.H, layer.W), rng):
        got.append(float(dxc[n, c, h, v]))
        ref.append(oracle.conv2d_bwd_data_at(dyo, wo, xo.shape, layer.stride, layer.pad, n, c, h, v))
    assert rel_l2(got, ref) <= 5e-3, ("bwd_data", name, rel_l2(got, ref))
    got, ref = [], []
    for (k, c, r, s) in _positions((layer.K, layer.C, layer.R, layer.S), rng):
        got.append(float(dwc[k, c, r, s]))
        ref.append(oracle.conv2d_bwd_filter_at(xo, dyo, wo.shape, layer.stride, layer.pad, k, c, r, s))
    assert rel_l2(got, ref) <= 5e-3, ("bwd_filter", name, rel_l2(got, ref))


def test_cheap_layers_full_size():
    """ReLU, BN and the 2x2 max-pool on the largest activation of the VGG-shaped configuration."""
    shape = (32, 64, 224, 224)
    x = wl.activation(shape, "bf16", seed=77)
    g = wl.activation(shape, "bf16", seed=78)
    xd, gd = x.cuda(), g.cuda()
    xo, go = f64(x), f64(g)
    out = torch.empty_like(xd)
    sn.sn_relu_fwd(xd, out)
    assert np.array_equal(f64(out), oracle.relu_fwd(xo))
    sn.sn_relu_bwd(xd, gd, out)
    assert np.array_equal(f64(out), oracle.relu_bwd(xo, go))
    gamma, beta = wl.bn_params(shape[1], 5)
    mean, invstd = torch.empty(shape[1], device="cuda"), torch.empty(shape[1], device="cuda")
    sn.sn_bn_fwd(xd, gamma.cuda(), beta.cuda(), out, mean, invstd)
    yo, mo, io = oracle.bn_fwd(xo, f64(gamma), f64(beta))
    assert rel_l2(f64(mean), mo) <= 1e-5 or np.linalg.norm(f64(mean) - mo) <= 1e-5
    assert rel_l2(f64(invstd), io) <= 1e-5
    assert rel_l2(f64(out), yo) <= 5e-3
    dgamma, dbeta = torch.empty(shape[1], device="cuda"), torch.empty(shape[1], device="cuda")
    sn.sn_bn_bwd(xd, gd, gamma.cuda(), mean, invstd, out, dgamma, dbeta)
    dxo, dgo, dbo = oracle.bn_bwd(xo, go, f64(gamma), f64(mean), f64(invstd))
    assert rel_l2(f64(dgamma), dgo) <= 1e-4 and rel_l2(f64(dbeta), dbo) <= 1e-4
    assert rel_l2(f64(out), dxo) <= 5e-3
    del yo, dxo
    r = torch.clamp(x.to(torch.float32), min=0).to(torch.bfloat16)
    rd = r.cuda()
    pooled = torch.empty((32, 64, 112, 112), dtype=torch.bfloat16, device="cuda")
    idx = torch.empty((32, 64, 112, 112), dtype=torch.int32, device="cuda")
    sn.sn_maxpool_fwd(rd, pooled, idx, (2, 2), (2, 2))
    po, pio = oracle.maxpool_fwd(f64(r), (2, 2), (2, 2), (0, 0))
    assert np.array_equal(idx.cpu().numpy(), pio)
    assert np.array_equal(f64(pooled), po)
    gp = wl.activation((32, 64, 112, 112), "bf16", seed=79)
    sn.sn_maxpool_bwd(gp.cuda(), idx, out, (2, 2), (2, 2))
    assert np.array_equal(f64(out), oracle.maxpool_bwd(f64(gp), pio, shape))


def test_fused_cheap_layers_full_size():
    """The one-call forms the benchmark step uses, on the largest activation of the VGG-shaped
    configuration: bit-identical to the separate calls (which the test above holds against the oracle)."""
    shape = (32, 64, 224, 224)
    N, C, H, W = shape
    xd = wl.activation(shape, "bf16", seed=77).cuda()
    gamma, beta = (t.cuda() for t in wl.bn_params(C, 5))
    new = lambda: torch.empty(C, device="cuda")
    # separate calls
    a, mean, invstd = torch.empty_like(xd), new(), new()
    sn.sn_bn_relu_fwd(xd, gamma, beta, a, mean, invstd)
    pooled_ref = torch.empty((N, C, H // 2, W // 2), dtype=torch.bfloat16, device="cuda")
    idx_ref = torch.empty((N, C, H // 2, W // 2), dtype=torch.int32, device="cuda")
    sn.sn_maxpool_fwd(a, pooled_ref, idx_ref, (2, 2), (2, 2))
    gp = wl.activation((N, C, H // 2, W // 2), "bf16", seed=79).cuda()
    g = torch.empty_like(xd)
    sn.sn_maxpool_bwd(gp, idx_ref, g, (2, 2), (2, 2))
    gr = torch.empty_like(xd)
    sn.sn_relu_bwd(a, g, gr)
    dx_ref, dg_ref, db_ref = torch.empty_like(xd), new(), new()
    sn.sn_bn_bwd(xd, gr, gamma, mean, invstd, dx_ref, dg_ref, db_ref)
    del g, gr
    # BN + ReLU backward from x alone
    g2 = torch.empty_like(xd)
    sn.sn_maxpool_bwd(gp, idx_ref, g2, (2, 2), (2, 2))
    dx, dg, db = torch.empty_like(xd), new(), new()
    sn.sn_bn_relu_bwd(xd, g2, gamma, beta, mean, invstd, dx, dg, db)
    torch.cuda.synchronize()
    assert torch.equal(dx, dx_ref) and torch.equal(dg, dg_ref) and torch.equal(db, db_ref)
    del g2
    # BN + ReLU + pool, forward and backward, and the forward from given statistics
    pooled, idx = torch.empty_like(pooled_ref), torch.empty_like(idx_ref)
    m2, i2 = new(), new()
    sn.sn_bn_relu_pool2_fwd(xd, gamma, beta, pooled, idx, m2, i2)
    dx.fill_(float("nan"))
    sn.sn_bn_relu_pool2_bwd(xd, gp, idx, gamma, beta, m2, i2, dx, dg, db)
    torch.cuda.synchronize()
    assert torch.equal(m2, mean) and torch.equal(i2, invstd)
    assert torch.equal(pooled, pooled_ref) and torch.equal(idx, idx_ref)
    assert torch.equal(dx, dx_ref) and torch.equal(dg, dg_ref) and torch.equal(db, db_ref)
    pooled.fill_(float("nan"))
    idx.fill_(-1)
    sn.sn_bn_relu_pool2_apply(xd, gamma, beta, mean, invstd, pooled, idx)
    a2 = torch.empty_like(xd)
    sn.sn_bn_apply(xd, gamma, beta, mean, invstd, a2, relu=True)
    torch.cuda.synchronize()
    assert torch.equal(pooled, pooled_ref) and torch.equal(idx, idx_ref) and torch.equal(a2, a)


@pytest.mark.parametrize("name", ["conv1_1", "conv1_2", "conv2_2", "conv4_1", "conv5_2"])
def test_conv_fwd_bn_stats_full_size(name):
    """CONV forward with the BN statistics of its output at the benchmark's sizes and plan: y as the
    plain call writes it, statistics within 1e-5 of the oracle's on sampled channels of the stored y."""
    cfg = wl.CONFIGS[3]
    N, dtype = cfg["N"], cfg["dtype"]
    li, layer = [(i, l) for i, l in enumerate(cfg["layers"]) if l.name == name][0]
    x, w, _ = wl.conv_inputs(layer, N, dtype, wl.layer_seed(3, li))
    P, Q = wl.out_hw(layer)
    shape = shape_of(layer, N, dtype, dtype)
    budget = max(b for b in cfg["budgets"] if b is not None)
    ws = torch.empty(budget, dtype=torch.uint8, device="cuda")
    xd, wd = x.cuda(), w.cuda()
    y_ref = torch.empty((N, layer.K, P, Q), dtype=torch.bfloat16, device="cuda")
    sn.sn_conv_autotune(sn.SN_CONV_FWD, xd, wd, y_ref, shape, ws, iters=1)
    sn.sn_conv2d_fwd(xd, wd, y_ref, shape, sn.SN_ALGO_AUTO, ws)
    y = torch.full_like(y_ref, float("nan"))
    mean, invstd = torch.empty(layer.K, device="cuda"), torch.empty(layer.K, device="cuda")
    scratch = torch.empty(sn.sn_conv_bn_stats_scratch_bytes(shape), dtype=torch.uint8, device="cuda")
    sn.sn_conv2d_fwd_bn_stats(xd, wd, y, shape, mean, invstd, scratch, sn.SN_ALGO_AUTO, ws)
    torch.cuda.synchronize()
    assert torch.equal(y, y_ref)
    ks = sorted({0, 1, layer.K // 2, layer.K - 1})
    ys = f64(y[:, ks])
    _, mo, io = oracle.bn_fwd(ys, np.ones(len(ks)), np.zeros(len(ks)), 1e-5)
    assert rel_l2(f64(mean[ks]), mo) <= 1e-5 or np.linalg.norm(f64(mean[ks]) - mo) <= 1e-6
    assert rel_l2(f64(invstd[ks]), io) <= 1e-5
