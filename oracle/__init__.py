"""ctypes wrapper of the CPU oracle (oracle/lags_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU library and its Python binding never
import this package, and this package never imports them.

Every function takes and returns numpy arrays on the host.  The arithmetic is
all in the C file; this module only marshals arguments.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lags_oracle.c")
_LIB = os.path.join(_HERE, "liblags_oracle.so")

CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared"]


def build(force=False):
    """Compile the oracle with gcc.  Returns the path of the shared library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Layer(ctypes.Structure):
    _fields_ = [("offset", ctypes.c_int64), ("d", ctypes.c_int64), ("rho", ctypes.c_double)]


def _bind(path):
    lib = ctypes.CDLL(path)
    f32p = ctypes.POINTER(ctypes.c_float)
    i32p = ctypes.POINTER(ctypes.c_int32)
    lp = ctypes.POINTER(_Layer)
    lib.oracle_topk_count.restype = ctypes.c_int64
    lib.oracle_topk_count.argtypes = [ctypes.c_int64, ctypes.c_double]
    lib.oracle_accumulate.restype = None
    lib.oracle_accumulate.argtypes = [f32p, f32p, ctypes.c_int64, ctypes.c_float, f32p]
    lib.oracle_sparsify_layer.restype = ctypes.c_int
    lib.oracle_sparsify_layer.argtypes = [f32p, f32p, ctypes.c_int64, ctypes.c_float,
                                          ctypes.c_int64, i32p, f32p]
    lib.oracle_sparsify_model.restype = ctypes.c_int
    lib.oracle_sparsify_model.argtypes = [lp, ctypes.c_int32, f32p, f32p, ctypes.c_float, i32p, f32p]
    lib.oracle_merge_sparse.restype = ctypes.c_int
    lib.oracle_merge_sparse.argtypes = [lp, ctypes.c_int32, i32p, f32p, ctypes.c_int32,
                                        ctypes.c_int64, f32p]
    lib.oracle_apply_sparse.restype = ctypes.c_int
    lib.oracle_apply_sparse.argtypes = [lp, ctypes.c_int32, i32p, f32p, ctypes.c_int32, ctypes.c_int64, f32p]
    lib.oracle_delta_monitor.restype = ctypes.c_int
    lib.oracle_delta_monitor.argtypes = [lp, ctypes.c_int32, f32p, ctypes.c_int64, i32p, f32p, ctypes.c_int32,
                                         ctypes.c_int64, ctypes.POINTER(ctypes.c_double)]
    return lib


def _f32(a):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _i32(a):
    assert a.dtype == np.int32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _layers(layers):
    arr = (_Layer * len(layers))()
    for i, (offset, d, rho) in enumerate(layers):
        arr[i].offset, arr[i].d, arr[i].rho = int(offset), int(d), float(rho)
    return arr


class OracleLib:
    """The oracle's functions over one compiled shared library."""

    def __init__(self, path=None):
        self._lib = _bind(path or build())

    def build(self):
        return build()

    def topk_count(self, d, rho):
        return int(self._lib.oracle_topk_count(int(d), float(rho)))

    def accumulate(self, grad, residual, lr):
        acc = np.empty_like(grad)
        self._lib.oracle_accumulate(_f32(grad), _f32(residual), grad.size, np.float32(lr), _f32(acc))
        return acc

    def sparsify_layer(self, grad, residual, lr, k):
        """Returns (idx int32[k], val float32[k]); `residual` is updated in place."""
        d = grad.size
        assert residual.size == d
        idx = np.empty(k, np.int32)
        val = np.empty(k, np.float32)
        rc = self._lib.oracle_sparsify_layer(_f32(grad), _f32(residual), d, np.float32(lr), int(k),
                                             _i32(idx), _f32(val))
        if rc:
            raise ValueError("oracle_sparsify_layer failed (rc=%d)" % rc)
        return idx, val

    def total_k(self, layers):
        return sum(self.topk_count(d, rho) for (_, d, rho) in layers)

    def sparsify_model(self, layers, grad_flat, residual_flat, lr):
        """layers: sequence of (offset, d, rho).  Returns (idx, val) of length sum k_l."""
        n = self.total_k(layers)
        idx = np.empty(n, np.int32)
        val = np.empty(n, np.float32)
        rc = self._lib.oracle_sparsify_model(_layers(layers), len(layers), _f32(grad_flat),
                                             _f32(residual_flat), np.float32(lr), _i32(idx), _f32(val))
        if rc:
            raise ValueError("oracle_sparsify_model failed (rc=%d)" % rc)
        return idx, val

    def merge_sparse(self, layers, idx, val, P, stride_k, update_flat):
        """idx/val: P blocks of pairs, block p at p*stride_k.  Overwrites every layer of update_flat."""
        rc = self._lib.oracle_merge_sparse(_layers(layers), len(layers), _i32(idx), _f32(val), int(P),
                                           int(stride_k), _f32(update_flat))
        if rc:
            raise ValueError("oracle_merge_sparse failed (rc=%d)" % rc)
        return update_flat


    def apply_sparse(self, layers, idx, val, P, stride_k, param_flat):
        """param_flat -= merged update, in place, for every element of every layer."""
        rc = self._lib.oracle_apply_sparse(_layers(layers), len(layers), _i32(idx), _f32(val), int(P),
                                           int(stride_k), _f32(param_flat))
        if rc:
            raise ValueError("oracle_apply_sparse failed (rc=%d)" % rc)
        return param_flat

    def delta_monitor(self, layers, residual_flat, res_stride, idx, val, P, stride_k):
        """float64[n_layers, 3]: numerator, ||sum_p x^p||^2, delta per layer."""
        out = np.empty((len(layers), 3), np.float64)
        rc = self._lib.oracle_delta_monitor(_layers(layers), len(layers), _f32(residual_flat), int(res_stride),
                                            _i32(idx), _f32(val), int(P), int(stride_k),
                                            out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
        if rc:
            raise ValueError("oracle_delta_monitor failed (rc=%d)" % rc)
        return out


_default = None


def _get():
    global _default
    if _default is None:
        _default = OracleLib()
    return _default


def topk_count(d, rho):
    return _get().topk_count(d, rho)


def accumulate(grad, residual, lr):
    return _get().accumulate(grad, residual, lr)


def sparsify_layer(grad, residual, lr, k):
    return _get().sparsify_layer(grad, residual, lr, k)


def total_k(layers):
    return _get().total_k(layers)


def sparsify_model(layers, grad_flat, residual_flat, lr):
    return _get().sparsify_model(layers, grad_flat, residual_flat, lr)


def merge_sparse(layers, idx, val, P, stride_k, update_flat):
    return _get().merge_sparse(layers, idx, val, P, stride_k, update_flat)


def apply_sparse(layers, idx, val, P, stride_k, param_flat):
    return _get().apply_sparse(layers, idx, val, P, stride_k, param_flat)


def delta_monitor(layers, residual_flat, res_stride, idx, val, P, stride_k):
    return _get().delta_monitor(layers, residual_flat, res_stride, idx, val, P, stride_k)
