"""ctypes binding of libhbmcal.so: plain streaming kernels of the streaming pass's shape, used by
bench.py to measure the practical HBM ceiling of this GPU.  Measurement aid, no method code."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhbmcal.so")
KINDS = {"copy": 0, "read": 1, "triad": 2, "write": 3}
BYTES_PER_ELEMENT = {"copy": 8.0, "read": 4.0, "triad": 12.0, "write": 4.0}
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libhbmcal.so is not built: run `python -m paper_1911_08727_amd.build`")
        import torch  # noqa: F401  (its HIP runtime must be the one that is mapped)
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        L.hbmcal_time.restype = ctypes.c_int
        L.hbmcal_time.argtypes = [ctypes.c_int, vp, vp, vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int, vp,
                                  ctypes.POINTER(ctypes.c_float)]
        _lib = L
    return _lib


def gbs(kind, a, b, sink, n_elems, reps, lds_pad, stream):
    """Average GB/s of kernel `kind` over n_elems floats of the torch tensors a, b."""
    ms = ctypes.c_float(0.0)
    rc = lib().hbmcal_time(KINDS[kind], ctypes.c_void_p(a.data_ptr()), ctypes.c_void_p(b.data_ptr()),
                           ctypes.c_void_p(sink.data_ptr()), int(n_elems), int(reps), int(lds_pad),
                           ctypes.c_void_p(stream.cuda_stream), ctypes.byref(ms))
    if rc != 0:
        raise RuntimeError("hbmcal_time failed (%d)" % rc)
    return BYTES_PER_ELEMENT[kind] * n_elems / (ms.value * 1e-3) / 1e9
