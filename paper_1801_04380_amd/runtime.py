"""Python names for the C ABI of include/sn_runtime.h (argument marshalling only): the memory pool,
the network's execution order, the memory used per step under the paper's techniques, and the
per-step workspace budgets handed to the CONV planner."""
import ctypes

from ._lib import ConvShape, load

SN_L_DATA, SN_L_CONV, SN_L_ACT, SN_L_LRN, SN_L_POOL, SN_L_BN, SN_L_FC, SN_L_DROPOUT, SN_L_SOFTMAX, SN_L_JOIN = range(10)
SN_MEM_BASELINE, SN_MEM_LIVENESS, SN_MEM_OFFLOAD, SN_MEM_RECOMPUTE = range(4)
SN_RECOMP_SPEED, SN_RECOMP_MEMORY, SN_RECOMP_COST_AWARE = range(3)
SN_POOL_BLOCK = 1024


class MemSummary(ctypes.Structure):
    """Mirror of sn_mem_summary."""
    _fields_ = [("peak_bytes", ctypes.c_size_t), ("peak_step", ctypes.c_int32), ("tensors", ctypes.c_int32),
                ("extra_forward", ctypes.c_int32), ("l_peak", ctypes.c_size_t)]


class ConvStepPlan(ctypes.Structure):
    """Mirror of sn_conv_step_plan."""
    _fields_ = [("layer", ctypes.c_int32), ("fwd_step", ctypes.c_int32), ("bwd_step", ctypes.c_int32),
                ("fwd_budget", ctypes.c_size_t), ("bwd_budget", ctypes.c_size_t),
                ("algo_fwd", ctypes.c_int32), ("algo_bwd_data", ctypes.c_int32), ("algo_bwd_filter", ctypes.c_int32),
                ("ws_fwd", ctypes.c_size_t), ("ws_bwd_data", ctypes.c_size_t), ("ws_bwd_filter", ctypes.c_size_t)]


_vp, _sz, _i = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
SIGNATURES = {
    "sn_pool_create": (_vp, [_sz]),
    "sn_pool_destroy": (None, [_vp]),
    "sn_pool_alloc": (_i, [_vp, _sz, ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(_sz)]),
    "sn_pool_free": (_i, [_vp, ctypes.c_uint64]),
    "sn_pool_used_bytes": (_sz, [_vp]),
    "sn_pool_peak_bytes": (_sz, [_vp]),
    "sn_pool_high_water": (_sz, [_vp]),
    "sn_pool_largest_free": (_sz, [_vp]),
    "sn_net_create": (_vp, []),
    "sn_net_destroy": (None, [_vp]),
    "sn_net_add_layer": (_i, [_vp, _i, _sz, ctypes.POINTER(_i), _i]),
    "sn_net_set_conv_shape": (_i, [_vp, _i, ctypes.POINTER(ConvShape)]),
    "sn_net_layers": (_i, [_vp]),
    "sn_net_route": (_i, [_vp, ctypes.POINTER(_i), _i]),
    "sn_net_steps": (_i, [_vp]),
    "sn_net_memory_trace": (_i, [_vp, _i, _i, ctypes.POINTER(_sz), ctypes.POINTER(ctypes.c_int32),
                                 ctypes.POINTER(MemSummary)]),
    "sn_net_step_budgets": (_i, [_vp, _i, _i, _sz, ctypes.POINTER(_sz)]),
    "sn_net_plan_convs": (_i, [_vp, _i, _i, _sz, ctypes.POINTER(ConvStepPlan), _i]),
}
_ready = False


def _lib():
    global _ready
    lib = load()
    if not _ready:
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _ready = True
    return lib


class Pool:
    def __init__(self, nbytes):
        self._p = _lib().sn_pool_create(nbytes)
        if not self._p:
            raise MemoryError("sn_pool_create")

    def close(self):
        if self._p:
            _lib().sn_pool_destroy(self._p)
            self._p = None

    def __del__(self):
        try:
            self.close()
        except Exception:      # interpreter shutdown: the library may be gone already
            pass

    def alloc(self, nbytes):
        """-> (id, offset), or None if no empty node is large enough."""
        ident, off = ctypes.c_uint64(), ctypes.c_size_t()
        st = _lib().sn_pool_alloc(self._p, nbytes, ctypes.byref(ident), ctypes.byref(off))
        if st == 3:
            return None
        if st != 0:
            raise ValueError("sn_pool_alloc returned %d" % st)
        return ident.value, off.value

    def free(self, ident):
        st = _lib().sn_pool_free(self._p, ident)
        if st != 0:
            raise ValueError("sn_pool_free returned %d" % st)

    used_bytes = property(lambda self: _lib().sn_pool_used_bytes(self._p))
    peak_bytes = property(lambda self: _lib().sn_pool_peak_bytes(self._p))
    high_water = property(lambda self: _lib().sn_pool_high_water(self._p))
    largest_free = property(lambda self: _lib().sn_pool_largest_free(self._p))


class Net:
    def __init__(self):
        self._n = _lib().sn_net_create()
        if not self._n:
            raise MemoryError("sn_net_create")

    def close(self):
        if self._n:
            _lib().sn_net_destroy(self._n)
            self._n = None

    def __del__(self):
        try:
            self.close()
        except Exception:      # interpreter shutdown: the library may be gone already
            pass

    def add(self, kind, out_bytes, prev=()):
        arr = (ctypes.c_int * len(prev))(*prev)
        ident = _lib().sn_net_add_layer(self._n, kind, out_bytes, arr, len(prev))
        if ident < 0:
            raise ValueError("sn_net_add_layer refused the layer")
        return ident

    def set_conv_shape(self, layer, shape):
        st = _lib().sn_net_set_conv_shape(self._n, layer, ctypes.byref(shape))
        if st != 0:
            raise ValueError("sn_net_set_conv_shape returned %d" % st)

    def route(self):
        cap = _lib().sn_net_layers(self._n)
        arr = (ctypes.c_int * max(cap, 1))()
        n = _lib().sn_net_route(self._n, arr, cap)
        if n < 0:
            raise ValueError("sn_net_route failed")
        return list(arr[:n])

    def steps(self):
        return _lib().sn_net_steps(self._n)

    def memory_trace(self, level, strategy=SN_RECOMP_COST_AWARE):
        n = self.steps()
        b, l, s = (ctypes.c_size_t * n)(), (ctypes.c_int32 * n)(), MemSummary()
        st = _lib().sn_net_memory_trace(self._n, level, strategy, b, l, ctypes.byref(s))
        if st != 0:
            raise ValueError("sn_net_memory_trace returned %d" % st)
        return dict(bytes=list(b), live=list(l), peak=s.peak_bytes, peak_step=s.peak_step, tensors=s.tensors,
                    extra=s.extra_forward, l_peak=s.l_peak)

    def step_budgets(self, level, strategy, capacity):
        n = self.steps()
        f = (ctypes.c_size_t * n)()
        st = _lib().sn_net_step_budgets(self._n, level, strategy, capacity, f)
        if st != 0:
            raise ValueError("sn_net_step_budgets returned %d" % st)
        return list(f)

    def plan_convs(self, level, strategy, capacity):
        cap = _lib().sn_net_layers(self._n)
        arr = (ConvStepPlan * max(cap, 1))()
        n = _lib().sn_net_plan_convs(self._n, level, strategy, capacity, arr, cap)
        if n < 0:
            raise ValueError("sn_net_plan_convs failed")
        return [{k: getattr(arr[i], k) for k, _ in ConvStepPlan._fields_} for i in range(n)]
