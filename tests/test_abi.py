"""CPU-only checks of the C ABI: the library loads, exports every symbol the
header declares, and its host-side logic (shape rule, argument checks, workspace
queries, planner) behaves as documented.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

import paper_1801_04380_amd as sn
from paper_1801_04380_amd import _lib

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "sn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sn_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = _lib.load()
    names = _declared_symbols()
    assert len(names) >= 16
    for name in names:
        assert hasattr(lib, name), name
        assert name in _lib.SIGNATURES, "binding lacks " + name
    assert lib.sn_version() == 1


def test_out_dim_floor_rule():
    assert sn.sn_out_dim(227, 0, 11, 4) == 55
    assert sn.sn_out_dim(55, 0, 3, 2) == 27
    assert sn.sn_out_dim(27, 0, 3, 2) == 13
    assert sn.sn_out_dim(56, 0, 1, 2) == 28      # floor, not ceil
    assert sn.sn_out_dim(56, 1, 3, 2) == 28
    assert sn.sn_out_dim(35, 0, 3, 2) == 17
    assert sn.sn_out_dim(2, 0, 3, 1) == 0        # window does not fit


def test_bad_arguments_are_refused_before_any_launch():
    lib = _lib.load()
    s = sn.conv_shape(2, 16, 16, 16, 16, 3, 3, (1, 1), (1, 1))
    one = ctypes.c_void_p(256)
    # null tensors
    assert lib.sn_conv2d_fwd(None, None, None, ctypes.byref(s), 0, None, 0, None) == 1
    # misaligned tensor pointer
    assert lib.sn_conv2d_fwd(ctypes.c_void_p(260), one, one, ctypes.byref(s), 0, None, 0, None) == 1
    # workspace bytes without a workspace, misaligned workspace
    assert lib.sn_conv2d_fwd(one, one, one, ctypes.byref(s), 0, None, 1024, None) == 1
    assert lib.sn_conv2d_fwd(one, one, one, ctypes.byref(s), 0, ctypes.c_void_p(128), 1024, None) == 1
    # named algorithm with too little workspace
    assert lib.sn_conv2d_fwd(one, one, one, ctypes.byref(s), sn.SN_ALGO_IM2COL_GEMM, one, 256, None) == 3
    # bad shapes
    for field, val in (("N", 0), ("stride_h", 0), ("pad_w", -1), ("in_dtype", 5), ("R", 40)):
        b = sn.conv_shape(2, 16, 16, 16, 16, 3, 3, (1, 1), (1, 1))
        setattr(b, field, val)
        assert lib.sn_conv2d_fwd(one, one, one, ctypes.byref(b), 0, None, 0, None) == 1, field
    # fp32 inputs cannot produce bf16 outputs
    b = sn.conv_shape(2, 16, 16, 16, 16, 3, 3, in_dtype=sn.SN_F32, out_dtype=sn.SN_BF16)
    assert lib.sn_conv2d_fwd(one, one, one, ctypes.byref(b), 0, None, 0, None) == 1
    # cheap layers
    assert lib.sn_relu_fwd(None, None, 10, 0, None) == 1
    assert lib.sn_relu_fwd(None, None, 0, 0, None) == 0          # empty tensor: nothing to do
    assert lib.sn_bn_fwd(one, one, one, one, one, one, 1, 1, 1, 1, 1e-5, 0, None) == 1   # y aliases x
    assert lib.sn_bn_relu_fwd(one, one, one, one, one, one, 1, 1, 1, 1, 1e-5, 0, None) == 1   # y aliases x
    two = ctypes.c_void_p(512)
    # the pair's backward needs beta to re-derive the ReLU gate; dx must alias none of its inputs
    assert lib.sn_bn_relu_bwd(one, two, one, None, one, one, ctypes.c_void_p(768), one, one, 1, 1, 1, 1, 0, None) == 1
    assert lib.sn_bn_relu_bwd(one, two, one, one, one, one, two, one, one, 1, 1, 1, 1, 0, None) == 1
    assert lib.sn_maxpool_fwd(one, one, one, 1, 1, 4, 4, 2, 2, 2, 2, 2, 0, 0, None) == 1  # pad >= window
    # CONV forward with the statistics for BN: needs its scratch, large enough
    s3 = sn.conv_shape(2, 16, 16, 16, 16, 3, 3, (1, 1), (1, 1))
    need = lib.sn_conv_bn_stats_scratch_bytes(ctypes.byref(s3))
    assert need >= 256 and need % 256 == 0
    assert lib.sn_conv_bn_stats_scratch_bytes(ctypes.byref(sn.conv_shape(0, 16, 16, 16, 16, 3, 3))) == 0
    assert lib.sn_conv2d_fwd_bn_stats(one, one, one, ctypes.byref(s3), 0, None, 0, one, one, 1e-5, None, 0, None) == 1
    assert lib.sn_conv2d_fwd_bn_stats(one, one, one, ctypes.byref(s3), 0, None, 0, one, one, 1e-5, one, need - 1, None) == 3
    assert lib.sn_conv2d_fwd_bn_stats(one, one, one, ctypes.byref(s3), 0, None, 0, one, None, 1e-5, one, need, None) == 1
    assert lib.sn_conv2d_fwd_bn_stats(one, one, one, ctypes.byref(s3), 0, None, 0, one, one, -1.0, one, need, None) == 1
    # BN from given statistics
    assert lib.sn_bn_apply(one, one, one, one, None, two, 1, 1, 1, 1, 0, 0, None) == 1
    assert lib.sn_bn_apply(one, one, one, one, one, two, 1, 1, 0, 1, 0, 0, None) == 1
    assert lib.sn_bn_apply(one, one, one, one, one, one, 1, 1, 1, 1, 0, 0, None) == 1    # y aliases x
    assert lib.sn_bn_relu_pool2_apply(one, one, one, one, one, two, ctypes.c_void_p(768), 1, 1, 5, 8, 1, None) == 2
    assert lib.sn_bn_relu_pool2_apply(one, one, one, one, one, two, two, 1, 1, 4, 8, 1, None) == 1
    # LRN: odd window of at most 9 channels, k > 0, no aliasing
    assert lib.sn_lrn_fwd(one, two, 1, 4, 2, 2, 4, 1e-4, 0.75, 2.0, 0, None) == 1
    assert lib.sn_lrn_fwd(one, two, 1, 4, 2, 2, 11, 1e-4, 0.75, 2.0, 0, None) == 2
    assert lib.sn_lrn_fwd(one, two, 1, 4, 2, 2, 5, 1e-4, 0.75, 0.0, 0, None) == 1
    assert lib.sn_lrn_fwd(one, one, 1, 4, 2, 2, 5, 1e-4, 0.75, 2.0, 0, None) == 1
    assert lib.sn_lrn_bwd(one, two, two, 1, 4, 2, 2, 5, 1e-4, 0.75, 2.0, 0, None) == 1
    assert lib.sn_lrn_bwd(one, None, two, 1, 4, 2, 2, 5, 1e-4, 0.75, 2.0, 0, None) == 1
    assert lib.sn_relu_lrn_fwd(one, one, 1, 4, 2, 2, 5, 1e-4, 0.75, 2.0, 0, None) == 1
    assert lib.sn_relu_lrn_fwd(one, two, 1, 4, 2, 2, 11, 1e-4, 0.75, 2.0, 0, None) == 2
    assert lib.sn_relu_lrn_bwd(one, two, two, 1, 4, 2, 2, 5, 1e-4, 0.75, 2.0, 0, None) == 1
    # BN + ReLU + 2x2 pool: odd sizes and rows too short for a vector access are for the separate calls
    three = ctypes.c_void_p(768)
    assert lib.sn_bn_relu_pool2_fwd(one, one, one, two, three, one, one, 1, 1, 5, 8, 1e-5, 1, None) == 2
    assert lib.sn_bn_relu_pool2_fwd(one, one, one, two, three, one, one, 1, 1, 14, 14, 1e-5, 1, None) == 2
    assert lib.sn_bn_relu_pool2_fwd(one, one, one, two, two, one, one, 1, 1, 4, 8, 1e-5, 1, None) == 1   # pooled aliases idx
    assert lib.sn_bn_relu_pool2_fwd(one, one, one, two, None, one, one, 1, 1, 4, 8, 1e-5, 1, None) == 1
    assert lib.sn_bn_relu_pool2_bwd(one, two, three, one, one, one, one, one, one, one, 1, 1, 4, 8, 1, None) == 1  # dx aliases x
    assert lib.sn_bn_relu_pool2_bwd(one, two, three, one, one, one, one, ctypes.c_void_p(1024), one, one, 1, 1, 4, 6, 1, None) == 2


def test_workspace_query():
    s = sn.conv_shape(2, 16, 16, 16, 16, 3, 3, (1, 1), (1, 1))
    assert sn.sn_conv_workspace_query(s, sn.SN_CONV_FWD, sn.SN_ALGO_DIRECT) == (0, 0)
    mn, pf = sn.sn_conv_workspace_query(s, sn.SN_CONV_FWD, sn.SN_ALGO_IM2COL_GEMM)
    # one image / the whole batch of the unfolded input: C*R*S*P*Q fp32 (288 KiB for the batch of 2)
    assert mn == 16 * 9 * 256 * 4 and pf == 2 * mn == 288 * 1024
    mn, pf = sn.sn_conv_workspace_query(s, sn.SN_CONV_BWD_FILTER, sn.SN_ALGO_STAGED)
    assert mn == pf and mn % 256 == 0 and mn >= 16 * 16 * 9 * 4
    b = sn.conv_shape(2, 16, 16, 16, 16, 3, 3, (1, 1), (1, 1), sn.SN_BF16, sn.SN_BF16)
    mnb, _ = sn.sn_conv_workspace_query(b, sn.SN_CONV_FWD, sn.SN_ALGO_IM2COL_GEMM)
    assert mnb == 16 * 9 * 256 * 2
    mnd, _ = sn.sn_conv_workspace_query(b, sn.SN_CONV_BWD_DATA, sn.SN_ALGO_IM2COL_GEMM)
    assert mnd == 16 * 9 * 256 * 4                # the column gradient is fp32
