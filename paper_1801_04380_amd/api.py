"""Python names for the C ABI of include/sn.h (argument marshalling only).

Tensors are torch CUDA (ROCm) tensors used as device memory; each call runs on
torch's current stream.  Nothing here computes anything.
"""
import ctypes

import torch

from ._lib import ConvShape, load

__all__ = [
    "SN_F32", "SN_BF16", "SN_CONV_FWD", "SN_CONV_BWD_DATA", "SN_CONV_BWD_FILTER",
    "SN_ALGO_AUTO", "SN_ALGO_DIRECT", "SN_ALGO_IM2COL_GEMM", "SN_ALGO_STAGED", "SN_ALGO_WINOGRAD", "ALGO_NAMES",
    "SnError", "conv_shape", "sn_out_dim", "sn_conv_workspace_query", "sn_conv_plan",
    "sn_planner_record", "sn_planner_clear", "sn_conv_autotune",
    "sn_conv2d_fwd", "sn_conv2d_bwd_data", "sn_conv2d_bwd_filter", "sn_conv2d_fwd_noalloc",
    "SN_NOALLOC_SCRATCH_BYTES",
    "sn_conv_bn_stats_scratch_bytes", "sn_conv2d_fwd_bn_stats", "sn_bn_apply", "sn_bn_relu_pool2_apply",
    "sn_relu_fwd", "sn_relu_bwd", "sn_bn_fwd", "sn_bn_relu_fwd", "sn_bn_bwd", "sn_bn_relu_bwd", "sn_bn_relu_pool2_fwd", "sn_bn_relu_pool2_bwd", "sn_lrn_fwd", "sn_lrn_bwd", "sn_relu_lrn_fwd", "sn_relu_lrn_bwd", "sn_maxpool_fwd", "sn_maxpool_bwd",
    "sn_measure_ceiling", "SN_CEIL_MFMA_BF16", "SN_CEIL_MFMA_F32", "SN_CEIL_COPY", "SN_CEIL_READ", "SN_CEIL_WRITE", "SN_CEIL_MFMA_BF16_FED",
]

SN_F32, SN_BF16 = 0, 1
SN_CONV_FWD, SN_CONV_BWD_DATA, SN_CONV_BWD_FILTER = 0, 1, 2
SN_ALGO_AUTO, SN_ALGO_DIRECT, SN_ALGO_IM2COL_GEMM, SN_ALGO_STAGED, SN_ALGO_WINOGRAD = -1, 0, 1, 2, 3
ALGO_NAMES = {SN_ALGO_AUTO: "auto", SN_ALGO_DIRECT: "direct", SN_ALGO_IM2COL_GEMM: "im2col_gemm",
              SN_ALGO_STAGED: "staged", SN_ALGO_WINOGRAD: "winograd"}
_STATUS = {1: "SN_ERR_BAD_ARG", 2: "SN_ERR_UNSUPPORTED", 3: "SN_ERR_WORKSPACE_TOO_SMALL", 4: "SN_ERR_LAUNCH"}


class SnError(RuntimeError):
    def __init__(self, call, status):
        super().__init__("%s returned %s" % (call, _STATUS.get(status, status)))
        self.status = status


def _check(call, status):
    if status != 0:
        raise SnError(call, status)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return SN_F32
    if t.dtype == torch.bfloat16:
        return SN_BF16
    raise TypeError("only float32 and bfloat16 tensors are supported, got %s" % t.dtype)


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def conv_shape(N, C, H, W, K, R, S, stride=(1, 1), pad=(0, 0), in_dtype=SN_F32, out_dtype=None):
    if out_dtype is None:
        out_dtype = in_dtype
    return ConvShape(N, C, H, W, K, R, S, stride[0], stride[1], pad[0], pad[1], in_dtype, out_dtype)


def sn_out_dim(size, pad, window, stride):
    return load().sn_out_dim(size, pad, window, stride)


def sn_conv_workspace_query(shape, direction, algo):
    """-> (min_bytes, preferred_bytes); raises SnError(SN_ERR_UNSUPPORTED) if the algorithm cannot run."""
    mn, pf = ctypes.c_size_t(), ctypes.c_size_t()
    _check("sn_conv_workspace_query",
           load().sn_conv_workspace_query(ctypes.byref(shape), direction, algo, ctypes.byref(mn), ctypes.byref(pf)))
    return mn.value, pf.value


def sn_conv_plan(shape, direction, budget_bytes):
    """-> (algo, bytes_used, predicted_ms or None)."""
    algo, used, ms = ctypes.c_int(), ctypes.c_size_t(), ctypes.c_float()
    _check("sn_conv_plan", load().sn_conv_plan(ctypes.byref(shape), direction, budget_bytes, ctypes.byref(algo),
                                               ctypes.byref(used), ctypes.byref(ms)))
    return algo.value, used.value, (ms.value if ms.value >= 0 else None)


def sn_planner_record(shape, direction, algo, workspace_bytes, ms):
    _check("sn_planner_record", load().sn_planner_record(ctypes.byref(shape), direction, algo, workspace_bytes, ms))


def sn_planner_clear():
    load().sn_planner_clear()


def _ws(workspace):
    if workspace is None:
        return None, 0
    return _ptr(workspace), workspace.numel() * workspace.element_size()


def sn_conv_autotune(direction, a, b, out, shape, workspace=None, iters=3):
    wp, wb = _ws(workspace)
    _check("sn_conv_autotune", load().sn_conv_autotune(direction, _ptr(a), _ptr(b), _ptr(out), ctypes.byref(shape),
                                                       wp, wb, iters, _stream()))


def sn_conv2d_fwd(x, w, y, shape, algo=SN_ALGO_AUTO, workspace=None):
    wp, wb = _ws(workspace)
    _check("sn_conv2d_fwd", load().sn_conv2d_fwd(_ptr(x), _ptr(w), _ptr(y), ctypes.byref(shape), algo, wp, wb,
                                                 _stream()))


SN_NOALLOC_SCRATCH_BYTES = 8 << 20


def sn_conv2d_fwd_noalloc(x, w, y, shape):
    _check("sn_conv2d_fwd_noalloc", load().sn_conv2d_fwd_noalloc(_ptr(x), _ptr(w), _ptr(y), ctypes.byref(shape),
                                                                 _stream()))


def sn_conv_bn_stats_scratch_bytes(shape):
    return int(load().sn_conv_bn_stats_scratch_bytes(ctypes.byref(shape)))


def sn_conv2d_fwd_bn_stats(x, w, y, shape, save_mean, save_invstd, scratch, algo=SN_ALGO_AUTO, workspace=None,
                           eps=1e-5):
    wp, wb = _ws(workspace)
    _check("sn_conv2d_fwd_bn_stats", load().sn_conv2d_fwd_bn_stats(
        _ptr(x), _ptr(w), _ptr(y), ctypes.byref(shape), algo, wp, wb, _ptr(save_mean), _ptr(save_invstd), eps,
        _ptr(scratch), scratch.numel() * scratch.element_size(), _stream()))


def sn_conv2d_bwd_data(dy, w, dx, shape, algo=SN_ALGO_AUTO, workspace=None):
    wp, wb = _ws(workspace)
    _check("sn_conv2d_bwd_data", load().sn_conv2d_bwd_data(_ptr(dy), _ptr(w), _ptr(dx), ctypes.byref(shape), algo,
                                                           wp, wb, _stream()))


def sn_conv2d_bwd_filter(x, dy, dw, shape, algo=SN_ALGO_AUTO, workspace=None):
    wp, wb = _ws(workspace)
    _check("sn_conv2d_bwd_filter", load().sn_conv2d_bwd_filter(_ptr(x), _ptr(dy), _ptr(dw), ctypes.byref(shape),
                                                               algo, wp, wb, _stream()))


def sn_relu_fwd(x, y):
    _check("sn_relu_fwd", load().sn_relu_fwd(_ptr(x), _ptr(y), x.numel(), _dtype_code(x), _stream()))


def sn_relu_bwd(x, dy, dx):
    _check("sn_relu_bwd", load().sn_relu_bwd(_ptr(x), _ptr(dy), _ptr(dx), x.numel(), _dtype_code(x), _stream()))


def sn_bn_fwd(x, gamma, beta, y, save_mean, save_invstd, eps=1e-5):
    N, C, H, W = x.shape
    _check("sn_bn_fwd", load().sn_bn_fwd(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(save_mean),
                                         _ptr(save_invstd), N, C, H, W, eps, _dtype_code(x), _stream()))


def sn_bn_relu_fwd(x, gamma, beta, y, save_mean, save_invstd, eps=1e-5):
    N, C, H, W = x.shape
    _check("sn_bn_relu_fwd", load().sn_bn_relu_fwd(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(save_mean),
                                                   _ptr(save_invstd), N, C, H, W, eps, _dtype_code(x), _stream()))


def sn_bn_apply(x, gamma, beta, mean, invstd, y, relu=False):
    N, C, H, W = x.shape
    _check("sn_bn_apply", load().sn_bn_apply(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(mean), _ptr(invstd), _ptr(y),
                                             N, C, H, W, int(relu), _dtype_code(x), _stream()))


def sn_bn_relu_pool2_apply(x, gamma, beta, mean, invstd, pooled, idx):
    N, C, H, W = x.shape
    _check("sn_bn_relu_pool2_apply", load().sn_bn_relu_pool2_apply(
        _ptr(x), _ptr(gamma), _ptr(beta), _ptr(mean), _ptr(invstd), _ptr(pooled), _ptr(idx), N, C, H, W,
        _dtype_code(x), _stream()))


def sn_bn_bwd(x, dy, gamma, save_mean, save_invstd, dx, dgamma, dbeta):
    N, C, H, W = x.shape
    _check("sn_bn_bwd", load().sn_bn_bwd(_ptr(x), _ptr(dy), _ptr(gamma), _ptr(save_mean), _ptr(save_invstd),
                                         _ptr(dx), _ptr(dgamma), _ptr(dbeta), N, C, H, W, _dtype_code(x),
                                         _stream()))


def sn_bn_relu_bwd(x, dy, gamma, beta, save_mean, save_invstd, dx, dgamma, dbeta):
    N, C, H, W = x.shape
    _check("sn_bn_relu_bwd", load().sn_bn_relu_bwd(_ptr(x), _ptr(dy), _ptr(gamma), _ptr(beta), _ptr(save_mean),
                                                   _ptr(save_invstd), _ptr(dx), _ptr(dgamma), _ptr(dbeta), N, C, H,
                                                   W, _dtype_code(x), _stream()))


def sn_bn_relu_pool2_fwd(x, gamma, beta, pooled, idx, save_mean, save_invstd, eps=1e-5):
    N, C, H, W = x.shape
    _check("sn_bn_relu_pool2_fwd", load().sn_bn_relu_pool2_fwd(
        _ptr(x), _ptr(gamma), _ptr(beta), _ptr(pooled), _ptr(idx), _ptr(save_mean), _ptr(save_invstd), N, C, H, W,
        eps, _dtype_code(x), _stream()))


def sn_bn_relu_pool2_bwd(x, dpooled, idx, gamma, beta, save_mean, save_invstd, dx, dgamma, dbeta):
    N, C, H, W = x.shape
    _check("sn_bn_relu_pool2_bwd", load().sn_bn_relu_pool2_bwd(
        _ptr(x), _ptr(dpooled), _ptr(idx), _ptr(gamma), _ptr(beta), _ptr(save_mean), _ptr(save_invstd), _ptr(dx),
        _ptr(dgamma), _ptr(dbeta), N, C, H, W, _dtype_code(x), _stream()))


def sn_lrn_fwd(x, y, size=5, alpha=1e-4, beta=0.75, k=2.0):
    N, C, H, W = x.shape
    _check("sn_lrn_fwd", load().sn_lrn_fwd(_ptr(x), _ptr(y), N, C, H, W, size, alpha, beta, k, _dtype_code(x),
                                           _stream()))


def sn_lrn_bwd(x, dy, dx, size=5, alpha=1e-4, beta=0.75, k=2.0):
    N, C, H, W = x.shape
    _check("sn_lrn_bwd", load().sn_lrn_bwd(_ptr(x), _ptr(dy), _ptr(dx), N, C, H, W, size, alpha, beta, k,
                                           _dtype_code(x), _stream()))


def sn_relu_lrn_fwd(x, y, size=5, alpha=1e-4, beta=0.75, k=2.0):
    N, C, H, W = x.shape
    _check("sn_relu_lrn_fwd", load().sn_relu_lrn_fwd(_ptr(x), _ptr(y), N, C, H, W, size, alpha, beta, k,
                                                     _dtype_code(x), _stream()))


def sn_relu_lrn_bwd(x, dy, dx, size=5, alpha=1e-4, beta=0.75, k=2.0):
    N, C, H, W = x.shape
    _check("sn_relu_lrn_bwd", load().sn_relu_lrn_bwd(_ptr(x), _ptr(dy), _ptr(dx), N, C, H, W, size, alpha, beta, k,
                                                     _dtype_code(x), _stream()))


SN_CEIL_MFMA_BF16, SN_CEIL_MFMA_F32, SN_CEIL_COPY, SN_CEIL_READ, SN_CEIL_WRITE, SN_CEIL_MFMA_BF16_FED = 0, 1, 2, 3, 4, 5


def sn_measure_ceiling(kind, buf, iters=5):
    """-> TFLOP/s (MFMA kinds) or GB/s (streaming kinds) on the device buf lives on."""
    val = ctypes.c_double()
    _check("sn_measure_ceiling", load().sn_measure_ceiling(kind, _ptr(buf), buf.numel() * buf.element_size(), iters,
                                                           _stream(), ctypes.byref(val)))
    return val.value


def sn_maxpool_fwd(x, y, idx, kernel, stride, pad=(0, 0)):
    N, C, H, W = x.shape
    _check("sn_maxpool_fwd", load().sn_maxpool_fwd(_ptr(x), _ptr(y), _ptr(idx), N, C, H, W, kernel[0], kernel[1],
                                                   stride[0], stride[1], pad[0], pad[1], _dtype_code(x),
                                                   _stream()))


def sn_maxpool_bwd(dy, idx, dx, kernel, stride, pad=(0, 0)):
    N, C, H, W = dx.shape
    _check("sn_maxpool_bwd", load().sn_maxpool_bwd(_ptr(dy), _ptr(idx), _ptr(dx), N, C, H, W, kernel[0], kernel[1],
                                                   stride[0], stride[1], pad[0], pad[1], _dtype_code(dx),
                                                   _stream()))
