"""Loads libsn_hip.so and declares the C ABI of include/sn.h for ctypes."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsn_hip.so")


class ConvShape(ctypes.Structure):
    """Mirror of sn_conv_shape."""
    _fields_ = [(n, ctypes.c_int32) for n in (
        "N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w",
        "in_dtype", "out_dtype")]


_vp, _sz, _i = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
_shape_p = ctypes.POINTER(ConvShape)
_conv_args = [_vp, _vp, _vp, _shape_p, _i, _vp, _sz, _vp]

# name -> (restype, argtypes); every symbol include/sn.h declares
SIGNATURES = {
    "sn_version": (_i, []),
    "sn_out_dim": (_i, [_i, _i, _i, _i]),
    "sn_conv_workspace_query": (_i, [_shape_p, _i, _i, ctypes.POINTER(_sz), ctypes.POINTER(_sz)]),
    "sn_conv_plan": (_i, [_shape_p, _i, _sz, ctypes.POINTER(_i), ctypes.POINTER(_sz),
                          ctypes.POINTER(ctypes.c_float)]),
    "sn_planner_record": (_i, [_shape_p, _i, _i, _sz, ctypes.c_float]),
    "sn_planner_clear": (None, []),
    "sn_conv_autotune": (_i, [_i, _vp, _vp, _vp, _shape_p, _vp, _sz, _i, _vp]),
    "sn_conv2d_fwd": (_i, _conv_args),
    "sn_conv2d_fwd_noalloc": (_i, [_vp, _vp, _vp, _shape_p, _vp]),
    "sn_conv_bn_stats_scratch_bytes": (_sz, [_shape_p]),
    "sn_conv2d_fwd_bn_stats": (_i, _conv_args[:-1] + [_vp, _vp, ctypes.c_float, _vp, _sz, _vp]),
    "sn_conv2d_bwd_data": (_i, _conv_args),
    "sn_conv2d_bwd_filter": (_i, _conv_args),
    "sn_relu_fwd": (_i, [_vp, _vp, _sz, _i, _vp]),
    "sn_relu_bwd": (_i, [_vp, _vp, _vp, _sz, _i, _vp]),
    "sn_bn_fwd": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, ctypes.c_float, _i, _vp]),
    "sn_bn_relu_fwd": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, ctypes.c_float, _i, _vp]),
    "sn_bn_apply": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp]),
    "sn_bn_relu_pool2_apply": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp]),
    "sn_bn_bwd": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp]),
    "sn_bn_relu_bwd": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp]),  # x, dy, gamma, beta, ...
    "sn_bn_relu_pool2_fwd": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, ctypes.c_float, _i, _vp]),
    "sn_bn_relu_pool2_bwd": (_i, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp]),
    "sn_lrn_fwd": (_i, [_vp, _vp, _i, _i, _i, _i, _i, ctypes.c_float, ctypes.c_float, ctypes.c_float, _i, _vp]),
    "sn_lrn_bwd": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, ctypes.c_float, ctypes.c_float, ctypes.c_float, _i, _vp]),
    "sn_relu_lrn_fwd": (_i, [_vp, _vp, _i, _i, _i, _i, _i, ctypes.c_float, ctypes.c_float, ctypes.c_float, _i, _vp]),
    "sn_relu_lrn_bwd": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, ctypes.c_float, ctypes.c_float, ctypes.c_float, _i, _vp]),
    "sn_measure_ceiling": (_i, [_i, _vp, _sz, _i, _vp, ctypes.POINTER(ctypes.c_double)]),
    "sn_maxpool_fwd": (_i, [_vp, _vp, _vp] + [_i] * 10 + [_i, _vp]),
    "sn_maxpool_bwd": (_i, [_vp, _vp, _vp] + [_i] * 10 + [_i, _vp]),
}

_lib = None


def load():
    """Load the HIP library; there is no fallback if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "%s is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                "(or python paper_1801_04380_amd/build.py) first" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib
