"""Helpers shared by the GPU parity tests: run one call of the HIP library on
host tensors and compare with the fp64 oracle fed the same (already rounded)
values."""
import numpy as np
import torch

import oracle
import paper_1801_04380_amd as sn

TOL = {"f32": 1e-5, "bf16": 5e-3}   # relative L2, fp32 path / bf16-input path
DT = {"f32": torch.float32, "bf16": torch.bfloat16}
CODE = {"f32": sn.SN_F32, "bf16": sn.SN_BF16}


def rel_l2(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = np.linalg.norm(want.ravel())
    num = np.linalg.norm((got - want).ravel())
    if den == 0.0:
        return 0.0 if num == 0.0 else np.inf
    return num / den


def elementwise_excess(got, want, tol, out_bf16=False):
    """The bound on every single element that goes beside the relative L2 (a norm alone lets one wrong
    element in 10^5 through): |got - want| <= 8 * tol * rms(want), plus half a bf16 unit of the element
    where the result is stored as bf16.  Returns the worst excess over the bound (<= 0 passes)."""
    got = np.asarray(got, dtype=np.float64).ravel()
    want = np.asarray(want, dtype=np.float64).ravel()
    if not np.isfinite(got).all():
        return np.inf
    rms = float(np.sqrt(np.mean(want * want))) if want.size else 0.0
    bound = 8 * tol * rms + (2.0 ** -8 * np.abs(want) if out_bf16 else 0.0)
    return float(np.max(np.abs(got - want) - bound)) if want.size else 0.0


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def shape_of(layer, N, dtype, out_dtype=None):
    return sn.conv_shape(N, layer.C, layer.H, layer.W, layer.K, layer.R, layer.S, layer.stride, layer.pad,
                         CODE[dtype], CODE[out_dtype or dtype])


def workspace(nbytes):
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device="cuda")


def run_conv(direction, a, b, out_shape, out_dtype, shape, algo, ws_bytes):
    """Run one conv call on the GPU; a, b are CPU tensors in storage dtype."""
    ad, bd = a.cuda(), b.cuda()
    # poison the output so that elements the kernel skips are caught
    out = torch.full(out_shape, float("nan"), dtype=out_dtype, device="cuda")
    ws = workspace(ws_bytes)
    fn = {sn.SN_CONV_FWD: sn.sn_conv2d_fwd, sn.SN_CONV_BWD_DATA: sn.sn_conv2d_bwd_data,
          sn.SN_CONV_BWD_FILTER: sn.sn_conv2d_bwd_filter}[direction]
    fn(ad, bd, out, shape, algo, ws)
    torch.cuda.synchronize()
    return out.cpu()
