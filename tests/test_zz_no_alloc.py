"""sn_conv2d_fwd_noalloc, the forward CONV for callers that cannot allocate: its workspace is a
fixed array inside the library.  It runs the kernels of sn_conv2d_fwd with SN_ALGO_STAGED, so the
outputs must be bit-identical; two calls in a row, the second on a smaller problem, share the array.
Also checked against the fp64 oracle (relative L2 <= 5e-3, bf16 inputs)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_1801_04380_amd as sn
from paper_1801_04380_amd import _lib
from paper_1801_04380_amd import workloads as wl
from _parity import f64, rel_l2

pytestmark = pytest.mark.gpu

# (N, C, H, W, K, R, S, pad): the second is smaller in every dimension
CASES = [(3, 80, 28, 28, 160, 3, 3, (1, 1)), (2, 24, 14, 14, 40, 3, 3, (1, 1))]


def _raw_call(x, w, y, shape):
    """Through the C ABI itself (ctypes), on torch's current stream."""
    lib = _lib.load()
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return lib.sn_conv2d_fwd_noalloc(ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(w.data_ptr()),
                                     ctypes.c_void_p(y.data_ptr()), ctypes.byref(shape), st)


def test_two_calls_in_a_row_match_the_workspace_entry_point():
    for i, (N, C, H, W, K, R, S, pad) in enumerate(CASES):
        layer = wl.Layer("t", C, H, W, K, R, S, (1, 1), pad, True, None, 1, False, None)
        x, w, _ = wl.conv_inputs(layer, N, "bf16", 4242 + i)
        shape = sn.conv_shape(N, C, H, W, K, R, S, (1, 1), pad, sn.SN_BF16, sn.SN_BF16)
        xd, wd = x.cuda(), w.cuda()
        P, Q = wl.out_hw(layer)
        mn, pf = sn.sn_conv_workspace_query(shape, sn.SN_CONV_FWD, sn.SN_ALGO_STAGED)
        assert mn <= sn.SN_NOALLOC_SCRATCH_BYTES
        ws = torch.empty(pf, dtype=torch.uint8, device="cuda")
        want = torch.full((N, K, P, Q), float("nan"), dtype=torch.bfloat16, device="cuda")
        sn.sn_conv2d_fwd(xd, wd, want, shape, sn.SN_ALGO_STAGED, ws)
        got = torch.full_like(want, float("nan"))
        assert _raw_call(xd, wd, got, shape) == 0
        torch.cuda.synchronize()
        assert not torch.isnan(got).any()
        assert torch.equal(got, want), "call %d differs from sn_conv2d_fwd(STAGED)" % i
        ref = oracle.conv2d_fwd(f64(x), f64(w), (1, 1), pad)
        assert rel_l2(f64(got), ref) <= 5e-3


def test_sizes_beyond_the_array_are_refused():
    # packed filter of 1024 x 1024 x 3 x 3 bf16 = 18 MiB > 8 MiB: refused, nothing launched
    shape = sn.conv_shape(1, 1024, 8, 8, 1024, 3, 3, (1, 1), (1, 1), sn.SN_BF16, sn.SN_BF16)
    x = torch.zeros((1, 1024, 8, 8), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((1024, 1024, 3, 3), dtype=torch.bfloat16, device="cuda")
    y = torch.full((1, 1024, 8, 8), 7.0, dtype=torch.bfloat16, device="cuda")
    assert _raw_call(x, w, y, shape) == 3
    # fp32 inputs have no STAGED kernel
    shape2 = sn.conv_shape(1, 16, 8, 8, 16, 3, 3, (1, 1), (1, 1), sn.SN_F32, sn.SN_F32)
    assert _raw_call(x, w, y, shape2) == 2
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())
