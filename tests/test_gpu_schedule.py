"""The budget generator feeding the kernels (Sec. 3.5): a small AlexNet-shaped network is scheduled
with sn_runtime.h under a device capacity a little above its peak, every CONV step gets the free
bytes of its step as its workspace budget, and the CONV calls run with exactly that much workspace:
results must match the fp64 oracle whatever the budget (the workspace never changes the function),
and the tight steps must end up on other algorithms than the roomy ones."""
import numpy as np
import pytest
import torch

import oracle
import paper_1801_04380_amd as sn
from paper_1801_04380_amd import runtime as rt
from paper_1801_04380_amd import workloads as wl
from _parity import TOL, elementwise_excess, f64, rel_l2, shape_of

pytestmark = pytest.mark.gpu

N = 8
L = wl.Layer
CONVS = [L("c1", 16, 31, 31, 64, 3, 3, (2, 2), (1, 1), False, None, 1, True, None),
         L("c2", 64, 16, 16, 96, 3, 3, (1, 1), (1, 1), True, None, 1, False, None),
         L("c3", 96, 8, 8, 128, 3, 3, (1, 1), (1, 1), True, None, 1, False, None),
         L("c4", 128, 8, 8, 128, 1, 1, (1, 1), (0, 0), True, None, 1, False, None)]


def _build():
    net = rt.Net()
    prev = net.add(rt.SN_L_DATA, N * 16 * 31 * 31 * 2)
    ids = {}
    for i, layer in enumerate(CONVS):
        P, Q = wl.out_hw(layer)
        out = N * layer.K * P * Q * 2
        prev = net.add(rt.SN_L_CONV, out, [prev])
        ids[prev] = layer
        net.set_conv_shape(prev, shape_of(layer, N, "bf16", "bf16"))
        if i < len(CONVS) - 1:     # the last CONV feeds the classifier directly: its backward is the peak step
            prev = net.add(rt.SN_L_BN, out, [prev])
            prev = net.add(rt.SN_L_ACT, out, [prev])
        if i == 1:
            prev = net.add(rt.SN_L_POOL, out // 4, [prev])
    prev = net.add(rt.SN_L_FC, N * 10 * 2, [prev])
    net.add(rt.SN_L_SOFTMAX, N * 10 * 2, [prev])
    return net, ids


def test_budgets_from_the_schedule_drive_the_conv_calls():
    net, ids = _build()
    sn.sn_planner_clear()
    level, strategy = rt.SN_MEM_LIVENESS, rt.SN_RECOMP_COST_AWARE
    trace = net.memory_trace(level, strategy)
    capacity = trace["peak"] + 4096            # almost nothing is free at the peak step
    plans = net.plan_convs(level, strategy, capacity)
    assert [p["layer"] for p in plans] == sorted(ids)
    budgets = sorted({p["fwd_budget"] for p in plans} | {p["bwd_budget"] for p in plans})
    assert budgets[0] < 8192 and budgets[-1] > (1 << 20)      # tight and roomy steps both occur
    algos = set()
    arena = torch.empty(max(budgets[-1], 256), dtype=torch.uint8, device="cuda")
    for p in plans:
        layer = ids[p["layer"]]
        x, w, dy = wl.conv_inputs(layer, N, "bf16", 9000 + p["layer"])
        shape = shape_of(layer, N, "bf16", "bf16")
        xo, wo, dyo = f64(x), f64(w), f64(dy)
        xd, wd, dyd = x.cuda(), w.cuda(), dy.cuda()
        P, Q = wl.out_hw(layer)
        runs = [(sn.sn_conv2d_fwd, xd, wd, torch.bfloat16, (N, layer.K, P, Q), p["fwd_budget"], p["algo_fwd"], p["ws_fwd"],
                 lambda: oracle.conv2d_fwd(xo, wo, layer.stride, layer.pad)),
                (sn.sn_conv2d_bwd_data, dyd, wd, torch.bfloat16, tuple(x.shape), p["bwd_budget"], p["algo_bwd_data"],
                 p["ws_bwd_data"], lambda: oracle.conv2d_bwd_data(dyo, wo, xo.shape, layer.stride, layer.pad)),
                (sn.sn_conv2d_bwd_filter, xd, dyd, torch.float32, tuple(w.shape), p["bwd_budget"], p["algo_bwd_filter"],
                 p["ws_bwd_filter"], lambda: oracle.conv2d_bwd_filter(xo, dyo, wo.shape, layer.stride, layer.pad))]
        for fn, a, b, odt, oshape, budget, algo, used, ref in runs:
            assert used <= budget
            ws = arena[:budget] if budget else None
            out = torch.full(oshape, float("nan"), dtype=odt, device="cuda")
            fn(a, b, out, shape, sn.SN_ALGO_AUTO, ws)          # the planner decides again, from the same budget
            torch.cuda.synchronize()
            want = ref()
            assert rel_l2(f64(out), want) <= TOL["bf16"], (layer.name, fn.__name__, budget, algo)
            assert elementwise_excess(f64(out), want, TOL["bf16"], odt == torch.bfloat16) <= 0
            algos.add(algo)
    assert sn.SN_ALGO_DIRECT in algos and sn.SN_ALGO_STAGED in algos
    net.close()
