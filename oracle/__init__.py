"""fp64 CPU oracle -- TEST INFRASTRUCTURE, not part of the product.

Thin ctypes/numpy front end to ``sn_oracle.c`` (plain-loop definitions of CONV
forward/backward and the ACT / BN / POOL layers that SuperNeurons, arXiv
1801.04380 Sec. 3.4-3.5, runs and replays).  Only tests, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package; it imports nothing
from the HIP library and the HIP library imports nothing from here.

All arrays are C-contiguous float64 (indices int32); shapes follow the paper's
NCHW tensors: x[N,C,H,W], w[K,C,R,S], y[N,K,P,Q].
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sn_oracle.c")
_LIB = os.path.join(_HERE, "libsn_oracle.so")


def build(force=False):
    """Compile sn_oracle.c with gcc (-O2, OpenMP over outer loops only)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall",
           "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None
_D = ctypes.POINTER(ctypes.c_double)
_I = ctypes.POINTER(ctypes.c_int32)


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.sn_oracle_conv2d_fwd_at.restype = ctypes.c_double
        _lib.sn_oracle_conv2d_bwd_data_at.restype = ctypes.c_double
        _lib.sn_oracle_conv2d_bwd_filter_at.restype = ctypes.c_double
        _lib.sn_oracle_out_dim.restype = ctypes.c_int
    return _lib


def _d(a):
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_D)


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def num_threads():
    """Threads the OpenMP loops will use (for the benchmark's report)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        return int(env.split(",")[0])
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def out_dim(size, pad, filt, stride):
    return int(_load().sn_oracle_out_dim(int(size), int(pad), int(filt), int(stride)))


def _geom(x_shape, w_shape, stride, pad):
    N, C, H, W = x_shape
    K, C2, R, S = w_shape
    assert C == C2
    return (N, C, H, W, K, R, S, stride[0], stride[1], pad[0], pad[1])


def conv2d_fwd(x, w, stride=(1, 1), pad=(0, 0)):
    x, w = _f64(x), _f64(w)
    g = _geom(x.shape, w.shape, stride, pad)
    P, Q = out_dim(g[2], g[9], g[5], g[7]), out_dim(g[3], g[10], g[6], g[8])
    y = np.empty((g[0], g[4], P, Q), dtype=np.float64)
    _load().sn_oracle_conv2d_fwd(_d(x), _d(w), _d(y), *map(ctypes.c_int, g))
    return y


def conv2d_bwd_data(dy, w, x_shape, stride=(1, 1), pad=(0, 0)):
    dy, w = _f64(dy), _f64(w)
    g = _geom(x_shape, w.shape, stride, pad)
    dx = np.empty(tuple(x_shape), dtype=np.float64)
    _load().sn_oracle_conv2d_bwd_data(_d(dy), _d(w), _d(dx), *map(ctypes.c_int, g))
    return dx


def conv2d_bwd_filter(x, dy, w_shape, stride=(1, 1), pad=(0, 0)):
    x, dy = _f64(x), _f64(dy)
    g = _geom(x.shape, w_shape, stride, pad)
    dw = np.empty(tuple(w_shape), dtype=np.float64)
    _load().sn_oracle_conv2d_bwd_filter(_d(x), _d(dy), _d(dw), *map(ctypes.c_int, g))
    return dw


def conv2d_fwd_at(x, w, stride, pad, n, k, p, q):
    g = _geom(x.shape, w.shape, stride, pad)
    return float(_load().sn_oracle_conv2d_fwd_at(_d(x), _d(w), *map(ctypes.c_int, g + (n, k, p, q))))


def conv2d_bwd_data_at(dy, w, x_shape, stride, pad, n, c, h, v):
    g = _geom(x_shape, w.shape, stride, pad)
    return float(_load().sn_oracle_conv2d_bwd_data_at(_d(dy), _d(w), *map(ctypes.c_int, g + (n, c, h, v))))


def conv2d_bwd_filter_at(x, dy, w_shape, stride, pad, k, c, r, s):
    g = _geom(x.shape, w_shape, stride, pad)
    return float(_load().sn_oracle_conv2d_bwd_filter_at(_d(x), _d(dy), *map(ctypes.c_int, g + (k, c, r, s))))


def _points(fn, a, b, g, coords):
    coords = np.ascontiguousarray(coords, dtype=np.int32).reshape(-1, 4)
    out = np.empty(coords.shape[0], dtype=np.float64)
    fn(_d(a), _d(b), *map(ctypes.c_int, g), coords.ctypes.data_as(_I), ctypes.c_size_t(coords.shape[0]), _d(out))
    return out


def conv2d_fwd_points(x, w, stride, pad, coords):
    """y at the listed (n, k, p, q); x, w float64 C-contiguous."""
    return _points(_load().sn_oracle_conv2d_fwd_points, x, w, _geom(x.shape, w.shape, stride, pad), coords)


def conv2d_bwd_data_points(dy, w, x_shape, stride, pad, coords):
    """dx at the listed (n, c, h, v)."""
    return _points(_load().sn_oracle_conv2d_bwd_data_points, dy, w, _geom(x_shape, w.shape, stride, pad), coords)


def conv2d_bwd_filter_points(x, dy, w_shape, stride, pad, coords):
    """dw at the listed (k, c, r, s)."""
    return _points(_load().sn_oracle_conv2d_bwd_filter_points, x, dy, _geom(x.shape, w_shape, stride, pad), coords)


def relu_fwd(x):
    x = _f64(x)
    y = np.empty_like(x)
    _load().sn_oracle_relu_fwd(_d(x), _d(y), ctypes.c_size_t(x.size))
    return y


def relu_bwd(x, dy):
    x, dy = _f64(x), _f64(dy)
    dx = np.empty_like(x)
    _load().sn_oracle_relu_bwd(_d(x), _d(dy), _d(dx), ctypes.c_size_t(x.size))
    return dx


def bn_fwd(x, gamma, beta, eps=1e-5):
    x, gamma, beta = _f64(x), _f64(gamma), _f64(beta)
    N, C, H, W = x.shape
    y = np.empty_like(x)
    mean = np.empty(C, dtype=np.float64)
    invstd = np.empty(C, dtype=np.float64)
    _load().sn_oracle_bn_fwd(_d(x), _d(gamma), _d(beta), _d(y), _d(mean), _d(invstd),
                             N, C, H, W, ctypes.c_double(eps))
    return y, mean, invstd


def bn_bwd(x, dy, gamma, save_mean, save_invstd):
    x, dy, gamma = _f64(x), _f64(dy), _f64(gamma)
    save_mean, save_invstd = _f64(save_mean), _f64(save_invstd)
    N, C, H, W = x.shape
    dx = np.empty_like(x)
    dgamma = np.empty(C, dtype=np.float64)
    dbeta = np.empty(C, dtype=np.float64)
    _load().sn_oracle_bn_bwd(_d(x), _d(dy), _d(gamma), _d(save_mean), _d(save_invstd),
                             _d(dx), _d(dgamma), _d(dbeta), N, C, H, W)
    return dx, dgamma, dbeta


def maxpool_fwd(x, kernel, stride, pad=(0, 0)):
    x = _f64(x)
    N, C, H, W = x.shape
    P, Q = out_dim(H, pad[0], kernel[0], stride[0]), out_dim(W, pad[1], kernel[1], stride[1])
    y = np.empty((N, C, P, Q), dtype=np.float64)
    idx = np.empty((N, C, P, Q), dtype=np.int32)
    _load().sn_oracle_maxpool_fwd(_d(x), _d(y), idx.ctypes.data_as(_I), N, C, H, W,
                                  kernel[0], kernel[1], stride[0], stride[1], pad[0], pad[1])
    return y, idx


def maxpool_bwd(dy, idx, x_shape):
    dy = _f64(dy)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    N, C, H, W = x_shape
    P, Q = dy.shape[2], dy.shape[3]
    dx = np.empty(tuple(x_shape), dtype=np.float64)
    _load().sn_oracle_maxpool_bwd(_d(dy), idx.ctypes.data_as(_I), _d(dx), N, C, H, W, P, Q)
    return dx


def lrn_fwd(x, size=5, alpha=1e-4, beta=0.75, k=2.0):
    x = _f64(x)
    N, C, H, W = x.shape
    y = np.empty_like(x)
    _load().sn_oracle_lrn_fwd(_d(x), _d(y), N, C, H, W, int(size), ctypes.c_double(alpha), ctypes.c_double(beta),
                              ctypes.c_double(k))
    return y


def lrn_bwd(x, dy, size=5, alpha=1e-4, beta=0.75, k=2.0):
    x, dy = _f64(x), _f64(dy)
    N, C, H, W = x.shape
    dx = np.empty_like(x)
    _load().sn_oracle_lrn_bwd(_d(x), _d(dy), _d(dx), N, C, H, W, int(size), ctypes.c_double(alpha),
                              ctypes.c_double(beta), ctypes.c_double(k))
    return dx
