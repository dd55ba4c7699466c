#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

One step = one pass of the whole hot path over one batch of a synthetic,
network-shaped workload (default: the VGG-16-shaped configuration, N = 32, bf16
in / fp32 accumulate): for every conv layer, CONV forward, BN forward, ReLU
forward and max-pool forward (the layers recomputation replays; unless --no-fuse
BN and the ReLU after it are one call, sn_bn_relu_fwd, and so are their backward
passes, sn_bn_relu_bwd; where a 2x2 pool follows, BN + ReLU + pool are one call
each way, sn_bn_relu_pool2_fwd / _bwd; and where a channel is too large for BN's
one-pass kernel the CONV leaves the batch statistics of its output,
sn_conv2d_fwd_bn_stats, and BN is one pass from them, sn_bn_apply /
sn_bn_relu_pool2_apply; without BN, a ReLU and the LRN after it are one call each
way, sn_relu_lrn_fwd / _bwd), then their backward
passes, CONV backward-data and CONV backward-filter, each CONV planned under the
given workspace budget.  Inputs are resident in HBM before the timed
region; autotuning happens before it too.

After the warm-up steps a few steps run with a pair of events around every call:
that gives the per-class breakdown and names the dominant class, and is not part
of the timed region (two hundred event records per step cost time of their own).
The timed region is exactly --steps steps with events only around the launches of
the dominant class, on the stream they are launched on.

Prints ONE JSON line: conv fwd+bwd TFLOP/s over the whole step time, the roofline
of the dominant kernel class from the events of the timed region, and the CPU
oracle timed on a bounded sample as a baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"bf16_mfma_tflops": 2500.0, "f32_mfma_tflops": 157.3, "hbm_gbs": 8000.0}

# HBM bytes per launch of an op class, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this
# command (profiles/bench_vgg16_n32_hbm_traffic.txt gives the runs, the calibration and the sums).
# Only for the workload and budget the counters were collected on, and only while the kernel sources
# are the ones they were collected on (TRAFFIC_KERNEL_SET = kernel_set_id() at that time); anything
# else reports null with a note.
TRAFFIC_KERNEL_SET = "2a590e1a4009"
MEASURED_TRAFFIC = {("cfg3_vgg16_n32", 2 << 30, "conv_bwd_filter"): 262e6,
                    # forward and backward-data run the same kernels: one figure for the 25 launches of both
                    ("cfg3_vgg16_n32", 2 << 30, "conv_fwd"): 146e6,
                    ("cfg3_vgg16_n32", 2 << 30, "conv_bwd_data"): 146e6}
KERNELS = {"conv_fwd": "conv_tile2_kernel / conv_tile_kernel (+ pack_filter9_kernel), smallc_fwd_kernel, pointwise_kernel (1x1)",
           "conv_bwd_data": "conv_tile2_kernel / conv_tile_kernel (+ pack_filter9_kernel), pointwise_kernel (1x1)",
           "conv_bwd_filter": "wgrad_rows_kernel / smallc_wgrad_kernel / pointwise_wgrad_kernel + reduce_partials4_kernel (STAGED) or fill_zero_kernel (DIRECT)"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=3, help="configuration number 1..5 (3 = VGG-16 N=32)")
    ap.add_argument("--budget-mib", type=float, default=None, help="workspace budget; default: the largest listed")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-autotune", action="store_true")
    ap.add_argument("--plan-file", default=None,
                    help="JSON of the planner's choices: written after autotuning if absent, loaded instead of "
                         "autotuning if present (a run under a counter-collecting profiler then launches the kernels "
                         "the plain run launched; the profiler's cost per dispatch skews the autotuner's timings)")
    ap.add_argument("--no-budget-sweep", action="store_true", help="skip the conv timing at the smaller budgets")
    ap.add_argument("--no-fuse", action="store_true", help="BN and ReLU as separate calls, forward and backward")
    ap.add_argument("--table-dtype", default=None, choices=["bf16", "f32"], help="--table only: run the workload's layers in this type")
    ap.add_argument("--table-batch", type=int, default=None, help="--table only: batch size instead of the workload's")
    ap.add_argument("--detail", default=None, help="write the per-layer table to this JSON file")
    ap.add_argument("--table", default=None,
                    help="instead of the step: time every layer x direction x algorithm of the workload, and the "
                         "cheap layers on every conv output, and write the table to this text file")
    return ap.parse_args()


class Op:
    """One call of the step with its algorithmic work, timed with a pair of events."""

    def __init__(self, key, layer, fn, flops=0.0, nbytes=0.0, nominal=0.0):
        self.key, self.layer, self.fn = key, layer, fn
        self.flops, self.nbytes, self.nominal = flops, nbytes, nominal
        self.ms = []
        self.ev = None


def kernel_set_id():
    """A short hash of the sources of the kernels the traffic figures are about (the stride-1 tile,
    few-channel and backward-filter kernels): tells a stale counter figure from a current one."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_1801_04380_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.startswith(("conv_tile", "conv_wgrad", "conv_smallc")) and name.endswith((".hip", ".h")):
            with open(os.path.join(d, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:12]


def measure_ceilings(buf):
    """What the plainest kernels reach on this GPU (sn_measure_ceiling), beside the datasheet peaks."""
    import paper_1801_04380_amd as sn
    kinds = {"mfma_bf16_tflops": sn.SN_CEIL_MFMA_BF16, "mfma_bf16_fed_tflops": sn.SN_CEIL_MFMA_BF16_FED,
             "mfma_f32_tflops": sn.SN_CEIL_MFMA_F32,
             "hbm_copy_gbs": sn.SN_CEIL_COPY, "hbm_read_gbs": sn.SN_CEIL_READ, "hbm_write_gbs": sn.SN_CEIL_WRITE}
    out = {k: sn.sn_measure_ceiling(v, buf, iters=5) for k, v in kinds.items()}
    out["buffer_bytes"] = buf.numel()
    return out


def build_ops(cfg_no, budget, autotune, fuse, plan_file=None):
    import torch

    import paper_1801_04380_amd as sn
    from paper_1801_04380_amd import workloads as wl

    cfg = wl.CONFIGS[cfg_no]
    N, dtype = cfg["N"], cfg["dtype"]
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    code = sn.SN_BF16 if dtype == "bf16" else sn.SN_F32
    b = 2 if dtype == "bf16" else 4
    dev = "cuda"
    ws = torch.empty(max(budget, 256), dtype=torch.uint8, device=dev) if budget else None
    wsbox = [ws]   # the workspace the conv calls are handed; main() swaps in smaller budgets
    fwd_ops, bwd_ops, plans = [], [], {}
    tune_ms = 0.0
    saved_plan = plan_out = None
    if plan_file and os.path.exists(plan_file):
        with open(plan_file) as f:
            saved_plan = json.load(f)
    elif plan_file and autotune:
        plan_out = {}
    for li, layer in enumerate(cfg["layers"]):
        x, w, _ = wl.conv_inputs(layer, N, dtype, wl.layer_seed(cfg_no, li))
        P, Q = wl.out_hw(layer)
        K, C = layer.K, layer.C
        shape = sn.conv_shape(N, C, layer.H, layer.W, K, layer.R, layer.S, layer.stride, layer.pad, code, code)
        xd, wd = x.to(dev), w.to(dev)
        del x, w
        y = torch.empty((N, K, P, Q), dtype=tdt, device=dev)
        dy = torch.empty_like(y)
        dx = torch.empty_like(xd)
        dw = torch.empty((K, C, layer.R, layer.S), dtype=torch.float32, device=dev)
        nominal, algo_flops = wl.conv_flops(layer, N)
        ex, ew, ey = xd.numel(), wd.numel(), y.numel()

        def conv_call(direction, a, bb, out, shape=shape):
            fn = {0: sn.sn_conv2d_fwd, 1: sn.sn_conv2d_bwd_data, 2: sn.sn_conv2d_bwd_filter}[direction]
            return lambda: fn(a, bb, out, shape, sn.SN_ALGO_AUTO, wsbox[0])

        # the gradient that reaches the conv comes from the cheap layers' backward below;
        # fill it once so the autotune runs on real values
        dy.copy_(wl.activation((N, K, P, Q), dtype, wl.layer_seed(cfg_no, li) + 7).to(dev))
        if saved_plan is not None:
            for d in (0, 1, 2):
                for algo, used, ms in saved_plan.get("%s|%d" % (layer.name, d), []):
                    sn.sn_planner_record(shape, d, algo, used, ms)
        elif autotune:
            t0 = time.time()
            for d, (a, bb, out) in {0: (xd, wd, y), 1: (dy, wd, dx), 2: (xd, dy, dw)}.items():
                sn.sn_conv_autotune(d, a, bb, out, shape, ws, iters=5)
            torch.cuda.synchronize()
            tune_ms += (time.time() - t0) * 1e3
        for d in (0, 1, 2):
            algo, used, ms = sn.sn_conv_plan(shape, d, budget)
            plans[(layer.name, d)] = (sn.ALGO_NAMES[algo], used, ms)
            if plan_out is not None:
                # the choice at every budget of the workload: enough to reproduce each of them
                picks = {sn.sn_conv_plan(shape, d, bb_) for bb_ in sorted({budget} | {x_ if x_ is not None else budget for x_ in cfg["budgets"]})}
                plan_out["%s|%d" % (layer.name, d)] = sorted([a_, u_, m_] for a_, u_, m_ in picks if m_ is not None)
        names = {0: "conv_fwd", 1: "conv_bwd_data", 2: "conv_bwd_filter"}
        byts = {0: (ex + ew) * b + ey * b, 1: (ey + ew) * b + ex * b, 2: (ex + ey) * b + ew * 4}
        cheap_f, cheap_b = [], []
        act_in = y
        E = y.numel()
        if cfg["bn"]:
            gamma, beta = (t.to(dev) for t in wl.bn_params(K, wl.layer_seed(cfg_no, li)))
            ybn = torch.empty_like(y)
            mean, invstd = torch.empty(K, device=dev), torch.empty(K, device=dev)
        # Where a channel of the output is too large for the one-pass BN kernel (which holds it in
        # registers), the CONV leaves the batch statistics of its output and the BN is one pass from
        # them; elsewhere taking them in the CONV costs more than BN's own single pass saves.
        conv_stats = cfg["bn"] and fuse and N * P * Q * b > 13 * 1024 * 16
        if conv_stats:
            scratch = torch.empty(max(sn.sn_conv_bn_stats_scratch_bytes(shape), 256), dtype=torch.uint8, device=dev)
            fwd_call = (lambda xd=xd, wd=wd, y=y, shape=shape, m=mean, i=invstd, sc=scratch:
                        sn.sn_conv2d_fwd_bn_stats(xd, wd, y, shape, m, i, sc, sn.SN_ALGO_AUTO, wsbox[0]))
        else:
            fwd_call = conv_call(0, xd, wd, y)
        for _ in range(layer.mult):
            fwd_ops.append(Op(names[0], layer.name, fwd_call, algo_flops, byts[0], nominal))
        if cfg["bn"]:
            dgamma, dbeta = torch.empty(K, device=dev), torch.empty(K, device=dev)
            g_bn = torch.empty_like(y)
        a = torch.empty_like(y)
        # BN + ReLU + 2x2 pool as one call each way where the pool's shape allows: the full-resolution
        # activation and its gradient are then never written
        pool_pair = (cfg["bn"] and fuse and layer.pool == ((2, 2), (2, 2)) and P % 2 == 0 and Q % 2 == 0
                     and Q % (8 // b) == 0)
        if pool_pair:
            pass
        elif cfg["bn"] and fuse:
            # BN and the ReLU after it in one pass over the tensor, from the statistics the CONV left:
            # 1 read + 1 write of E elements is all the pair needs
            cheap_f.append(Op("bn_relu_fwd", layer.name,
                              (lambda y=y, ga=gamma, be=beta, o=a, m=mean, i=invstd: sn.sn_bn_apply(y, ga, be, m, i, o, relu=True))
                              if conv_stats else
                              (lambda y=y, ga=gamma, be=beta, o=a, m=mean, i=invstd: sn.sn_bn_relu_fwd(y, ga, be, o, m, i)),
                              nbytes=2 * E * b))
        else:
            if cfg["bn"]:
                cheap_f.append(Op("bn_fwd", layer.name,
                                  lambda y=y, ga=gamma, be=beta, o=ybn, m=mean, i=invstd: sn.sn_bn_fwd(y, ga, be, o, m, i),
                                  nbytes=2 * E * b))
                act_in = ybn
            # ReLU and the LRN after it in one pass each way (no BN in between): the ReLU output is never written
            relu_lrn = bool(fuse and layer.lrn and not cfg["bn"])
            if not relu_lrn:
                cheap_f.append(Op("relu_fwd", layer.name, lambda s=act_in, o=a: sn.sn_relu_fwd(s, o), nbytes=2 * E * b))
        g_a = torch.empty_like(y)
        pool_src, pool_grad = a, g_a
        relu_lrn = bool(fuse and layer.lrn and not cfg["bn"] and not pool_pair)
        if layer.lrn and not pool_pair:
            # LRN between the ReLU and the pool; its backward needs its input and the gradient only
            a_l, g_l = torch.empty_like(y), torch.empty_like(y)
            if relu_lrn:
                cheap_f.append(Op("relu_lrn_fwd", layer.name, lambda s=y, o=a_l, p=layer.lrn: sn.sn_relu_lrn_fwd(s, o, *p),
                                  nbytes=2 * E * b))
            else:
                cheap_f.append(Op("lrn_fwd", layer.name, lambda s=a, o=a_l, p=layer.lrn: sn.sn_lrn_fwd(s, o, *p),
                                  nbytes=2 * E * b))
            pool_src, pool_grad = a_l, g_l
        if layer.pool:
            kernel, stride = layer.pool
            PP, QQ = sn.sn_out_dim(P, 0, kernel[0], stride[0]), sn.sn_out_dim(Q, 0, kernel[1], stride[1])
            pooled = torch.empty((N, K, PP, QQ), dtype=tdt, device=dev)
            idx = torch.empty((N, K, PP, QQ), dtype=torch.int32, device=dev)
            g_pool = wl.activation((N, K, PP, QQ), dtype, wl.layer_seed(cfg_no, li) + 9).to(dev)
            Eo = pooled.numel()
        if pool_pair:
            cheap_f.append(Op("bn_relu_pool_fwd", layer.name,
                              (lambda y=y, ga=gamma, be=beta, o=pooled, ix=idx, m=mean, i=invstd:
                               sn.sn_bn_relu_pool2_apply(y, ga, be, m, i, o, ix)) if conv_stats else
                              (lambda y=y, ga=gamma, be=beta, o=pooled, ix=idx, m=mean, i=invstd:
                               sn.sn_bn_relu_pool2_fwd(y, ga, be, o, ix, m, i)), nbytes=E * b + Eo * (b + 4)))
            cheap_b.append(Op("bn_relu_pool_bwd", layer.name,
                              lambda y=y, g=g_pool, ix=idx, ga=gamma, be=beta, m=mean, i=invstd, o=dy, dg=dgamma, db=dbeta:
                              sn.sn_bn_relu_pool2_bwd(y, g, ix, ga, be, m, i, o, dg, db),
                              nbytes=Eo * (b + 4) + 2 * E * b))
        elif layer.pool:
            cheap_f.append(Op("maxpool_fwd", layer.name,
                              lambda s=pool_src, o=pooled, i=idx, k=kernel, st=stride: sn.sn_maxpool_fwd(s, o, i, k, st),
                              nbytes=E * b + Eo * (b + 4)))
            cheap_b.append(Op("maxpool_bwd", layer.name,
                              lambda g=g_pool, i=idx, o=pool_grad, k=kernel, st=stride: sn.sn_maxpool_bwd(g, i, o, k, st),
                              nbytes=Eo * (b + 4) + E * b))
        else:
            pool_grad.copy_(dy)
        if relu_lrn:
            cheap_b.append(Op("relu_lrn_bwd", layer.name,
                              lambda s=y, g=g_l, o=dy, p=layer.lrn: sn.sn_relu_lrn_bwd(s, g, o, *p), nbytes=3 * E * b))
        elif layer.lrn and not pool_pair:
            cheap_b.append(Op("lrn_bwd", layer.name,
                              lambda s=a, g=g_l, o=g_a, p=layer.lrn: sn.sn_lrn_bwd(s, g, o, *p), nbytes=3 * E * b))
        if pool_pair:
            pass
        elif cfg["bn"] and fuse:
            # ReLU backward and BN backward in one call: reads x and the gradient, writes dx (the
            # ReLU gate is re-derived from x)
            cheap_b.append(Op("bn_relu_bwd", layer.name,
                              lambda y=y, g=g_a, ga=gamma, be=beta, m=mean, i=invstd, o=dy, dg=dgamma, db=dbeta:
                              sn.sn_bn_relu_bwd(y, g, ga, be, m, i, o, dg, db), nbytes=3 * E * b))
        elif relu_lrn:
            pass
        else:
            relu_grad_out = g_bn if cfg["bn"] else dy
            cheap_b.append(Op("relu_bwd", layer.name, lambda s=a, g=g_a, o=relu_grad_out: sn.sn_relu_bwd(s, g, o),
                              nbytes=3 * E * b))
            if cfg["bn"]:
                cheap_b.append(Op("bn_bwd", layer.name,
                                  lambda y=y, g=g_bn, ga=gamma, m=mean, i=invstd, o=dy, dg=dgamma, db=dbeta:
                                  sn.sn_bn_bwd(y, g, ga, m, i, o, dg, db), nbytes=3 * E * b))
        for _ in range(layer.mult):
            fwd_ops.extend(cheap_f)
        layer_bwd = []
        for _ in range(layer.mult):
            layer_bwd.extend(cheap_b)
            if not layer.first:  # the gradient of the image is not needed in training
                layer_bwd.append(Op(names[1], layer.name, conv_call(1, dy, wd, dx), algo_flops, byts[1], nominal))
            layer_bwd.append(Op(names[2], layer.name, conv_call(2, xd, dy, dw), algo_flops, byts[2], nominal))
        bwd_ops = layer_bwd + bwd_ops  # backward visits the layers in reverse
    if plan_out is not None:
        with open(plan_file, "w") as f:
            json.dump(plan_out, f, indent=0, sort_keys=True)
    return cfg, fwd_ops + bwd_ops, plans, tune_ms, wsbox


def layer_table(cfg_no, budget, path, dtype_override=None, batch_override=None):
    """Per layer x direction x algorithm (at its least and its preferred workspace, the latter capped
    by the budget): median and minimum of 20 launches after 5 warm-up launches, each between a pair
    of events.  Cheap layers: every call on every conv output, rotating through three sets of
    buffers so that the working set of consecutive launches exceeds the 256 MB last-level cache."""
    import torch

    import paper_1801_04380_amd as sn
    from paper_1801_04380_amd import workloads as wl

    cfg = wl.CONFIGS[cfg_no]
    N, dtype, dev = batch_override or cfg["N"], dtype_override or cfg["dtype"], torch.device("cuda:0")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    code = sn.SN_BF16 if dtype == "bf16" else sn.SN_F32
    b = 2 if dtype == "bf16" else 4
    peak = PEAK["bf16_mfma_tflops"] if dtype == "bf16" else PEAK["f32_mfma_tflops"]
    ws = torch.empty(max(budget, 256), dtype=torch.uint8, device=dev)

    def timed(fns):
        """fns: the same call on rotating buffer sets; -> (median, min) ms over 20 launches."""
        for i in range(5):
            fns[i % len(fns)]()
        ev = []
        for i in range(20):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fns[i % len(fns)]()
            e1.record()
            ev.append((e0, e1))
        torch.cuda.synchronize()
        t = sorted(a.elapsed_time(c) for a, c in ev)
        return (t[9] + t[10]) / 2, t[0]

    out = ["%s, N = %d, %s, workspace budget %d MiB; times in us (median / min of 20 launches); TFLOP/s and %% of the"
           % (cfg["name"], N, dtype, budget >> 20),
           "dense MFMA peak (%.0f TFLOP/s) from algorithmic FLOPs and the median; GB/s and %% of 8 TB/s from the" % peak,
           "compulsory bytes of the call and the median.  F/B: algorithmic FLOPs per compulsory byte; roof: what bounds the",
           "call at that intensity (mfma above %.0f F/B, else hbm at 8 TB/s x F/B) and the share of that roof reached."
           % (peak * 1e12 / (PEAK["hbm_gbs"] * 1e9)), "",
           "%-10s %-10s %-12s %10s %9s %9s %8s %6s %7s %5s %7s" % ("layer", "direction", "algorithm", "ws MiB", "median", "min",
                                                                  "TFLOP/s", "peak", "F/B", "roof", "of roof")]
    names = {0: "forward", 1: "bwd-data", 2: "bwd-filter"}
    cheap = []
    for li, layer in enumerate(cfg["layers"]):
        x, w, dy = wl.conv_inputs(layer, N, dtype, wl.layer_seed(cfg_no, li))
        xd, wd, dyd = x.to(dev), w.to(dev), dy.to(dev)
        K = layer.K
        P, Q = wl.out_hw(layer)
        shape = sn.conv_shape(N, layer.C, layer.H, layer.W, K, layer.R, layer.S, layer.stride, layer.pad, code, code)
        y, dx = torch.empty((N, K, P, Q), dtype=tdt, device=dev), torch.empty_like(xd)
        dw = torch.empty(tuple(w.shape), dtype=torch.float32, device=dev)
        flops = wl.conv_flops(layer, N)[1]
        ex, ew, ey = xd.numel(), wd.numel(), y.numel()
        cbytes = {0: (ex + ew) * b + ey * b, 1: (ey + ew) * b + ex * b, 2: (ex + ey) * b + ew * 4}
        for d, (fn, a, bb, o) in {0: (sn.sn_conv2d_fwd, xd, wd, y), 1: (sn.sn_conv2d_bwd_data, dyd, wd, dx),
                                  2: (sn.sn_conv2d_bwd_filter, xd, dyd, dw)}.items():
            if d == 1 and layer.first:
                continue
            for algo in (sn.SN_ALGO_DIRECT, sn.SN_ALGO_STAGED, sn.SN_ALGO_IM2COL_GEMM, sn.SN_ALGO_WINOGRAD):
                try:
                    mn, pf = sn.sn_conv_workspace_query(shape, d, algo)
                except sn.SnError:
                    continue
                for used in sorted({mn, min(pf, budget)}):
                    if used < mn or used > budget:
                        continue
                    wsv = ws[:used] if used else None
                    med, lo = timed([lambda: fn(a, bb, o, shape, algo, wsv)])
                    tf = flops / (med * 1e-3) / 1e12
                    ai = flops / cbytes[d]
                    hbm_roof = ai * PEAK["hbm_gbs"] * 1e9 / 1e12
                    roof = min(peak, hbm_roof)
                    out.append("%-10s %-10s %-12s %10.1f %9.1f %9.1f %8.1f %5.1f%% %7.0f %5s %6.1f%%"
                               % (layer.name, names[d], sn.ALGO_NAMES[algo], used / 2 ** 20, med * 1e3, lo * 1e3, tf,
                                  100 * tf / peak, ai, "mfma" if peak <= hbm_roof else "hbm", 100 * tf / roof))
        cheap.append((layer, (N, K, P, Q)))
        del xd, wd, dyd, y, dx, dw
    out += ["", "%-10s %-22s %12s %9s %9s %8s %6s" % ("layer", "call", "MB moved", "median", "min", "GB/s", "of HBM")]
    seen = set()
    for layer, shp in cheap:
        if (shp, layer.pool, layer.lrn) in seen:
            continue
        seen.add((shp, layer.pool, layer.lrn))
        E = shp[0] * shp[1] * shp[2] * shp[3]
        sets = max(1, min(3, int(600e6 // (3 * E * b)) or 1)) if 3 * E * b < 600e6 else 3
        bufs = [[wl.activation(shp, dtype, 40 + i).to(dev) for i in range(2)] + [torch.empty(shp, dtype=tdt, device=dev) for _ in range(2)]
                for _ in range(sets)]
        gamma, beta = (t.to(dev) for t in wl.bn_params(shp[1], 1))
        stat = [torch.empty(shp[1], device=dev) for _ in range(4)]
        calls = [("relu_fwd", 2, lambda s: sn.sn_relu_fwd(s[0], s[2])),
                 ("relu_bwd", 3, lambda s: sn.sn_relu_bwd(s[0], s[1], s[2]))]
        if cfg["bn"]:
            calls += [("bn_fwd", 2, lambda s: sn.sn_bn_fwd(s[0], gamma, beta, s[2], stat[0], stat[1])),
                      ("bn_relu_fwd", 2, lambda s: sn.sn_bn_relu_fwd(s[0], gamma, beta, s[2], stat[0], stat[1])),
                      ("bn_apply (+relu)", 2, lambda s: sn.sn_bn_apply(s[0], gamma, beta, stat[0], stat[1], s[2], relu=True)),
                      ("bn_bwd", 3, lambda s: sn.sn_bn_bwd(s[0], s[1], gamma, stat[0], stat[1], s[2], stat[2], stat[3])),
                      ("bn_relu_bwd", 3, lambda s: sn.sn_bn_relu_bwd(s[0], s[1], gamma, beta, stat[0], stat[1], s[2], stat[2], stat[3]))]
        if layer.lrn:
            calls += [("lrn_fwd", 2, lambda s: sn.sn_lrn_fwd(s[0], s[2], *layer.lrn)),
                      ("lrn_bwd", 3, lambda s: sn.sn_lrn_bwd(s[0], s[1], s[2], *layer.lrn))]
        for cname, passes, f in calls:
            med, lo = timed([(lambda s=s_: f(s)) for s_ in bufs])
            mb = passes * E * b
            out.append("%-10s %-22s %12.1f %9.1f %9.1f %8.0f %5.1f%%" % (layer.name, cname, mb / 1e6, med * 1e3, lo * 1e3,
                                                                        mb / (med * 1e-3) / 1e9, 100 * mb / (med * 1e-3) / 1e9 / PEAK["hbm_gbs"]))
        if layer.pool:
            kernel, stride = layer.pool
            PP, QQ = sn.sn_out_dim(shp[2], 0, kernel[0], stride[0]), sn.sn_out_dim(shp[3], 0, kernel[1], stride[1])
            pooled = [torch.empty((shp[0], shp[1], PP, QQ), dtype=tdt, device=dev) for _ in range(sets)]
            idx = [torch.empty((shp[0], shp[1], PP, QQ), dtype=torch.int32, device=dev) for _ in range(sets)]
            gp = wl.activation((shp[0], shp[1], PP, QQ), dtype, 50).to(dev)
            Eo = pooled[0].numel()
            pc = [("maxpool_fwd", E * b + Eo * (b + 4), lambda i: sn.sn_maxpool_fwd(bufs[i][0], pooled[i], idx[i], kernel, stride)),
                  ("maxpool_bwd", Eo * (b + 4) + E * b, lambda i: sn.sn_maxpool_bwd(gp, idx[i], bufs[i][2], kernel, stride))]
            if cfg["bn"] and kernel == (2, 2) and stride == (2, 2) and shp[2] % 2 == 0 and shp[3] % (8 // b) == 0:
                pc += [("bn_relu_pool2_fwd", E * b + Eo * (b + 4),
                        lambda i: sn.sn_bn_relu_pool2_fwd(bufs[i][0], gamma, beta, pooled[i], idx[i], stat[0], stat[1])),
                       ("bn_relu_pool2_bwd", Eo * (b + 4) + 2 * E * b,
                        lambda i: sn.sn_bn_relu_pool2_bwd(bufs[i][0], gp, idx[i], gamma, beta, stat[0], stat[1], bufs[i][2],
                                                          stat[2], stat[3]))]
            for cname, mb, f in pc:
                med, lo = timed([(lambda i=i_: f(i)) for i_ in range(sets)])
                out.append("%-10s %-22s %12.1f %9.1f %9.1f %8.0f %5.1f%%" % (layer.name, cname, mb / 1e6, med * 1e3, lo * 1e3,
                                                                            mb / (med * 1e-3) / 1e9, 100 * mb / (med * 1e-3) / 1e9 / PEAK["hbm_gbs"]))
        del bufs
    with open(path, "w") as f:
        f.write("\n".join(out) + "\n")
    print("\n".join(out))


def cpu_baseline(cfg_no):
    """The fp64 oracle, as it stands, on a bounded sample: the most expensive layers of the
    workload (conv cost is linear in N, so a reduced batch where a layer alone would take too
    long), all three directions, until about 600 GFLOP of fp64 loops have run."""
    import oracle
    from paper_1801_04380_amd import workloads as wl

    cfg = wl.CONFIGS[cfg_no]
    layers = sorted(cfg["layers"], key=lambda l: -wl.conv_flops(l, 1)[0])
    budget, flops, dt, parts = 600e9, 0.0, 0.0, []
    for layer in layers[:2]:
        per_img = wl.conv_flops(layer, 1)[0]
        n = int(max(1, min(cfg["N"], round(budget / 2 / (3 * per_img)))))
        x, w, dy = wl.conv_inputs(layer, n, cfg["dtype"], 1)
        xo, wo, dyo = (t.double().numpy() for t in (x, w, dy))
        oracle.conv2d_fwd(xo[:1, :, :8, :8].copy(), wo, layer.stride, layer.pad)  # load the library
        t0 = time.time()
        oracle.conv2d_fwd(xo, wo, layer.stride, layer.pad)
        oracle.conv2d_bwd_data(dyo, wo, xo.shape, layer.stride, layer.pad)
        oracle.conv2d_bwd_filter(xo, dyo, wo.shape, layer.stride, layer.pad)
        dt += time.time() - t0
        flops += 3 * wl.conv_flops(layer, n)[1]
        parts.append("%s (C=%d K=%d %dx%d, %dx%d filter) at N=%d of %d"
                     % (layer.name, layer.C, layer.K, layer.H, layer.W, layer.R, layer.S, n, cfg["N"]))
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%s %s, fwd+bwd-data+bwd-filter, fp64, %.1f s" % (cfg["name"], " and ".join(parts), dt)}


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_1801_04380_amd as sn
    from paper_1801_04380_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    cfg = wl.CONFIGS[args.workload]
    budgets = [b for b in cfg["budgets"] if b]
    if args.budget_mib is not None:
        budget = int(args.budget_mib * (1 << 20))
    else:
        budget = max(budgets) if budgets else 64 << 20
    if args.table:
        layer_table(args.workload, budget, args.table, args.table_dtype, args.table_batch)
        return
    cfg, ops, plans, tune_ms, wsbox = build_ops(args.workload, budget, not args.no_autotune, not args.no_fuse, args.plan_file)
    stream = torch.cuda.current_stream()

    def step(timed_keys):
        """One pass of the hot path; ops whose class is in timed_keys get a pair of events."""
        for op in ops:
            if timed_keys is None or op.key in timed_keys:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                op.fn()
                e1.record(stream)
                op.ev = (op.ev or []) + [(e0, e1)]
            else:
                op.fn()

    def collect(robust=False):
        # an Op object appears once per occurrence in the step; shared objects (mult > 1) hold all their events
        # robust: every launch of an op counts with the op's median time -- in the breakdown pass, where
        # the host records two events per call and now and then falls behind the GPU, a pair of events
        # then also spans the GPU's wait for the next call to arrive
        seen, table = set(), {}
        for op in ops:
            if id(op) in seen or not op.ev:
                continue
            seen.add(id(op))
            times = [a.elapsed_time(bb) for a, bb in op.ev]
            if robust:
                med = sorted(times)[len(times) // 2]
                times = [med] * len(times)
            k = table.setdefault(op.key, dict(ms=0.0, launches=0, flops=0.0, nbytes=0.0, nominal=0.0, layers={}))
            k["ms"] += sum(times)
            k["launches"] += len(times)
            k["flops"] += op.flops * len(times)
            k["nominal"] += op.nominal * len(times)
            k["nbytes"] += op.nbytes * len(times)
            lay = k["layers"].setdefault(op.layer, dict(ms=0.0, launches=0, flops=op.flops, nbytes=op.nbytes))
            lay["ms"] += sum(times)
            lay["launches"] += len(times)
            op.ev = None
        return table

    for _ in range(args.warmup):
        step(set())
    # per-class breakdown: a pass of its own with events around every op (the events cost time, so
    # it is not the timed region); it also says which class is the dominant one
    BREAKDOWN_STEPS = 3
    torch.cuda.synchronize()
    for _ in range(BREAKDOWN_STEPS):
        step(None)
    torch.cuda.synchronize()
    by_key = collect(robust=True)
    dom = max(by_key, key=lambda k: by_key[k]["ms"])
    # the timed region: exactly args.steps steps, events only around the launches of the dominant class
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step({dom})
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    d = collect()[dom]

    # the other budgets of the workload (Sec. 3.5: less free memory, slower algorithms): the conv calls
    # alone, handed a smaller slice of the same workspace; the planner falls back by itself
    per_budget = {}
    full_ws = wsbox[0]
    for bb in sorted({x for x in cfg["budgets"] if x is not None} | {budget}):   # None = no limit: the default budget stands for it
        if bb > budget or args.no_budget_sweep:
            continue
        wsbox[0] = None if bb == 0 else full_ws[:bb]
        conv_ops = [op for op in ops if op.key.startswith("conv_")]
        for op in conv_ops:
            op.fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(3):
            for op in conv_ops:
                op.fn()
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 3
        fl = sum(op.flops for op in conv_ops)
        peak = PEAK["bf16_mfma_tflops"] if cfg["dtype"] == "bf16" else PEAK["f32_mfma_tflops"]
        per_budget[str(bb)] = {"conv_ms_per_step": ms, "conv_tflops": fl / (ms * 1e-3) / 1e12,
                               "frac_mfma_peak": fl / (ms * 1e-3) / 1e12 / peak}
    wsbox[0] = full_ws

    conv_keys = [k for k in by_key if k.startswith("conv_")]
    conv_flops_step = sum(by_key[k]["flops"] for k in conv_keys) / BREAKDOWN_STEPS
    conv_ms_step = sum(by_key[k]["ms"] for k in conv_keys) / BREAKDOWN_STEPS
    cheap_keys = [k for k in by_key if not k.startswith("conv_")]
    cheap_bytes_step = sum(by_key[k]["nbytes"] for k in cheap_keys) / BREAKDOWN_STEPS
    cheap_ms_step = sum(by_key[k]["ms"] for k in cheap_keys) / BREAKDOWN_STEPS
    replay_keys = [k for k in cheap_keys if k.endswith("_fwd")]
    replay_gbs = (sum(by_key[k]["nbytes"] for k in replay_keys) / max(sum(by_key[k]["ms"] for k in replay_keys), 1e-9)
                  / 1e6)
    value = conv_flops_step / (wall_ms * 1e-3) / 1e12

    avg_ms = d["ms"] / d["launches"]
    if dom.startswith("conv_"):
        peak = PEAK["bf16_mfma_tflops"] if cfg["dtype"] == "bf16" else PEAK["f32_mfma_tflops"]
        achieved = d["flops"] / d["launches"] / (avg_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                "traffic": None}
    else:
        achieved = d["nbytes"] / d["launches"] / (avg_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK["hbm_gbs"], "unit": "GB/s",
                "frac": achieved / PEAK["hbm_gbs"], "traffic": None}
    roof["traffic"] = MEASURED_TRAFFIC.get((cfg["name"], budget, dom))
    if roof["traffic"] is not None and kernel_set_id() != TRAFFIC_KERNEL_SET:
        roof["traffic"] = None
        roof["traffic_note"] = "the kernel sources changed since the counters in profiles/ were taken"
    # the device's own ceilings, on a buffer far beyond the memory-side cache
    cbuf = full_ws if (full_ws is not None and full_ws.numel() >= (1 << 30)) else torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    ceilings = measure_ceilings(cbuf)
    roof["peak_measured"] = (ceilings["mfma_bf16_tflops" if cfg["dtype"] == "bf16" else "mfma_f32_tflops"]
                             if roof["bound"] == "mfma" else ceilings["hbm_copy_gbs"])
    roof.update({"kernel": dom, "hip_kernels": KERNELS.get(dom, dom), "launches_per_step": d["launches"] / args.steps,
                 "avg_launch_ms": avg_ms, "algorithmic_bytes_per_launch": d["nbytes"] / d["launches"]})

    breakdown = {}
    for k, v in sorted(by_key.items()):
        e = {"ms_per_step": v["ms"] / BREAKDOWN_STEPS}
        if v["flops"]:
            e["tflops"] = v["flops"] / (v["ms"] * 1e-3) / 1e12
            e["frac_mfma_peak"] = e["tflops"] / (PEAK["bf16_mfma_tflops"] if cfg["dtype"] == "bf16"
                                                 else PEAK["f32_mfma_tflops"])
        else:
            e["gbs"] = v["nbytes"] / (v["ms"] * 1e-3) / 1e9
            e["frac_hbm_peak"] = e["gbs"] / PEAK["hbm_gbs"]
        breakdown[k] = e

    out = {
        "metric": "conv fwd+bwd TFLOP/s (% MFMA peak) per workspace budget; recompute GB/s",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": cfg["name"], "batch": cfg["N"], "workspace_budget_bytes": budget,
                   "layers": len(cfg["layers"]), "ops_per_step": len(ops)},
        "conv_only_tflops": conv_flops_step / (conv_ms_step * 1e-3) / 1e12,
        "conv_frac_mfma_peak": conv_flops_step / (conv_ms_step * 1e-3) / 1e12
        / (PEAK["bf16_mfma_tflops"] if cfg["dtype"] == "bf16" else PEAK["f32_mfma_tflops"]),
        "recompute_gbs": replay_gbs,
        "recompute_ms_per_step": sum(by_key[k]["ms"] for k in replay_keys) / BREAKDOWN_STEPS, "cheap_layers_gbs": cheap_bytes_step / (cheap_ms_step * 1e-3) / 1e9,
        "autotune_ms": tune_ms, "conv_per_budget": per_budget,
        "roofline": roof, "ceilings": ceilings, "breakdown": breakdown,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload)
    if args.detail:
        detail = {"plans": {"%s/%d" % k: v for k, v in plans.items()},
                  "layers": {k: v["layers"] for k, v in by_key.items()}}
        for k, v in detail["layers"].items():
            for name, lay in v.items():
                t = lay["ms"] / lay["launches"]
                lay["avg_ms"] = t
                if lay["flops"]:
                    lay["tflops"] = lay["flops"] / (t * 1e-3) / 1e12
                lay["gbs"] = lay["nbytes"] / (t * 1e-3) / 1e9
        os.makedirs(os.path.dirname(os.path.abspath(args.detail)), exist_ok=True)
        with open(args.detail, "w") as f:
            json.dump(detail, f, indent=1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
