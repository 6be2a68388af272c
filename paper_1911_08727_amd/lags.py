"""Thin ctypes binding of liblags.so: same names as include/lags.h, argument
marshalling only.  Torch tensors are used for device memory and streams; every
step of the method runs inside the library's HIP kernels.  There is no CPU
fallback: if the library is missing the import of a symbol fails loudly.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblags.so")

LAGS_OK, LAGS_EINVAL, LAGS_ENOMEM, LAGS_EHIP, LAGS_ECAPACITY = 0, -1, -2, -3, -4


class LayerDesc(ctypes.Structure):
    _fields_ = [("offset", ctypes.c_int64), ("d", ctypes.c_int64), ("rho", ctypes.c_double)]


class AllgatherModel(ctypes.Structure):
    _fields_ = [("alpha", ctypes.c_double), ("beta", ctypes.c_double), ("P", ctypes.c_int32)]


_lib = None


def lib():
    """Load liblags.so (built beforehand by paper_1911_08727_amd.build); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("liblags.so is not built: run `python -m paper_1911_08727_amd.build` "
                               "(there is no fallback path)")
        # torch ships its own HIP runtime; it must be the one already mapped when liblags.so
        # resolves libamdhip64, or the process ends up with two runtimes and no usable device
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, f32, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_double
        L.lags_topk_count.restype, L.lags_topk_count.argtypes = i64, [i64, dbl]
        L.lags_create.restype, L.lags_create.argtypes = ctypes.c_int, [ctypes.POINTER(vp), ctypes.c_int]
        L.lags_destroy.restype, L.lags_destroy.argtypes = ctypes.c_int, [vp]
        L.lags_table_create.restype = ctypes.c_int
        L.lags_table_create.argtypes = [vp, ctypes.POINTER(LayerDesc), i32, ctypes.POINTER(vp)]
        L.lags_table_destroy.restype, L.lags_table_destroy.argtypes = ctypes.c_int, [vp]
        L.lags_table_num_layers.restype, L.lags_table_num_layers.argtypes = i32, [vp]
        L.lags_table_total_k.restype, L.lags_table_total_k.argtypes = i64, [vp]
        L.lags_table_k.restype, L.lags_table_k.argtypes = i64, [vp, i32]
        L.lags_table_out_offset.restype, L.lags_table_out_offset.argtypes = i64, [vp, i32]
        L.lags_sparsify_layer.restype = ctypes.c_int
        L.lags_sparsify_layer.argtypes = [vp, vp, vp, i64, f32, i64, vp, vp, vp]
        L.lags_sparsify_layer_noalloc.restype = ctypes.c_int
        L.lags_sparsify_layer_noalloc.argtypes = [ctypes.c_int, vp, vp, i64, f32, i64, vp, vp, vp]
        L.lags_noalloc_max_elements.restype, L.lags_noalloc_max_elements.argtypes = i64, []
        L.lags_sparsify_model.restype = ctypes.c_int
        L.lags_sparsify_model.argtypes = [vp, vp, vp, vp, f32, vp, vp, vp]
        L.lags_merge_sparse.restype = ctypes.c_int
        L.lags_merge_sparse.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp]
        L.lags_strerror.restype, L.lags_strerror.argtypes = ctypes.c_char_p, [ctypes.c_int]
        L.lags_apply_sparse.restype = ctypes.c_int
        L.lags_apply_sparse.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp]
        L.lags_delta_monitor.restype = ctypes.c_int
        L.lags_delta_monitor.argtypes = [vp, vp, vp, i64, vp, vp, i32, i64, vp, vp]
        L.lags_last_routes.restype = ctypes.c_int
        L.lags_last_routes.argtypes = [vp, vp, ctypes.POINTER(i32), i32]
        L.lags_debug_fallback_chain.restype, L.lags_debug_fallback_chain.argtypes = ctypes.c_int, [vp, ctypes.c_int]
        L.lags_debug_scratch_info.restype = ctypes.c_int
        L.lags_debug_scratch_info.argtypes = [vp, ctypes.c_int, ctypes.POINTER(vp), ctypes.POINTER(i64),
                                              ctypes.POINTER(i64)]
        L.lags_debug_poison_scratch.restype, L.lags_debug_poison_scratch.argtypes = ctypes.c_int, [vp, vp]
        L.lags_profile_enable.restype, L.lags_profile_enable.argtypes = ctypes.c_int, [vp, ctypes.c_int]
        L.lags_profile_enable_kernel.restype = ctypes.c_int
        L.lags_profile_enable_kernel.argtypes = [vp, ctypes.c_int]
        L.lags_profile_num_kernels.restype, L.lags_profile_num_kernels.argtypes = ctypes.c_int, []
        L.lags_profile_kernel_name.restype, L.lags_profile_kernel_name.argtypes = ctypes.c_char_p, [ctypes.c_int]
        L.lags_profile_read.restype = ctypes.c_int
        L.lags_profile_read.argtypes = [vp, ctypes.c_int, ctypes.POINTER(dbl), ctypes.POINTER(i64)]
        L.lags_profile_reset.restype, L.lags_profile_reset.argtypes = ctypes.c_int, [vp]
        L.lags_profile_kernel_elements.restype = i64
        L.lags_profile_kernel_elements.argtypes = [vp, ctypes.c_int]
        L.lags_allgather_seconds.restype = dbl
        L.lags_allgather_seconds.argtypes = [ctypes.POINTER(AllgatherModel), i64]
        L.lags_adaptive_ratios.restype = ctypes.c_int
        L.lags_adaptive_ratios.argtypes = [ctypes.POINTER(AllgatherModel), ctypes.POINTER(i64),
                                           ctypes.POINTER(dbl), ctypes.POINTER(dbl), i32, dbl,
                                           ctypes.POINTER(i64), ctypes.POINTER(dbl)]
        _lib = L
    return _lib


class LagsError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, lib().lags_strerror(code).decode(), code))


def _check(code, where):
    if code != LAGS_OK:
        raise LagsError(code, where)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def lags_topk_count(d, rho):
    return int(lib().lags_topk_count(int(d), float(rho)))


def lags_sparsify_layer_noalloc(device, grad, residual, lr, k, out_idx, out_val, stream=None):
    _check(lib().lags_sparsify_layer_noalloc(int(device), _ptr(grad), _ptr(residual), grad.numel(), float(lr),
                                             int(k), _ptr(out_idx), _ptr(out_val), _stream(stream)),
           "lags_sparsify_layer_noalloc")


def lags_noalloc_max_elements():
    return int(lib().lags_noalloc_max_elements())


def lags_allgather_seconds(alpha, beta, P, k):
    net = AllgatherModel(float(alpha), float(beta), int(P))
    return float(lib().lags_allgather_seconds(ctypes.byref(net), int(k)))


def lags_adaptive_ratios(alpha, beta, P, d, t_comp, t_spar, c_u):
    """Host lists in, (k list, rho list) out."""
    n = len(d)
    net = AllgatherModel(float(alpha), float(beta), int(P))
    dd = (ctypes.c_int64 * n)(*[int(x) for x in d])
    tc = (ctypes.c_double * n)(*[float(x) for x in t_comp])
    ts = (ctypes.c_double * n)(*[float(x) for x in t_spar])
    k = (ctypes.c_int64 * n)()
    rho = (ctypes.c_double * n)()
    _check(lib().lags_adaptive_ratios(ctypes.byref(net), dd, tc, ts, n, float(c_u), k, rho), "lags_adaptive_ratios")
    return list(k), list(rho)


class Table:
    """Handle of a prepared layer table (lags_table_create / lags_table_destroy)."""

    def __init__(self, ctx, layers):
        self.ctx = ctx
        arr = (LayerDesc * len(layers))()
        for i, (offset, d, rho) in enumerate(layers):
            arr[i].offset, arr[i].d, arr[i].rho = int(offset), int(d), float(rho)
        h = ctypes.c_void_p(0)
        _check(lib().lags_table_create(ctx.handle, arr, len(layers), ctypes.byref(h)), "lags_table_create")
        self.handle = h
        self.n = len(layers)

    @property
    def total_k(self):
        return int(lib().lags_table_total_k(self.handle))

    def k(self, l):
        return int(lib().lags_table_k(self.handle, l))

    def out_offset(self, l):
        return int(lib().lags_table_out_offset(self.handle, l))

    def kernel_elements(self):
        """{kernel name: layer elements one launch covers} for this table."""
        out = {}
        for kid in range(lib().lags_profile_num_kernels()):
            n = int(lib().lags_profile_kernel_elements(self.handle, kid))
            if n > 0:
                out[lib().lags_profile_kernel_name(kid).decode()] = n
        return out

    def destroy(self):
        if self.handle:
            lib().lags_table_destroy(self.handle)
            self.handle = None


class Context:
    """Handle of a library context (lags_create / lags_destroy) on one HIP device."""

    def __init__(self, device=0):
        h = ctypes.c_void_p(0)
        _check(lib().lags_create(ctypes.byref(h), int(device)), "lags_create")
        self.handle = h
        self.device = device

    def table(self, layers):
        return Table(self, layers)

    def lags_sparsify_layer(self, grad, residual, lr, k, out_idx, out_val, stream=None):
        _check(lib().lags_sparsify_layer(self.handle, _ptr(grad), _ptr(residual), grad.numel(), float(lr),
                                         int(k), _ptr(out_idx), _ptr(out_val), _stream(stream)),
               "lags_sparsify_layer")

    def lags_sparsify_model(self, table, grad_flat, residual_flat, lr, out_idx, out_val, stream=None):
        _check(lib().lags_sparsify_model(self.handle, table.handle, _ptr(grad_flat), _ptr(residual_flat),
                                         float(lr), _ptr(out_idx), _ptr(out_val), _stream(stream)),
               "lags_sparsify_model")

    def lags_merge_sparse(self, table, idx, val, P, stride_k, update_flat, stream=None):
        _check(lib().lags_merge_sparse(self.handle, table.handle, _ptr(idx), _ptr(val), int(P), int(stride_k),
                                       _ptr(update_flat), _stream(stream)), "lags_merge_sparse")

    def lags_apply_sparse(self, table, idx, val, P, stride_k, param_flat, stream=None):
        _check(lib().lags_apply_sparse(self.handle, table.handle, _ptr(idx), _ptr(val), int(P), int(stride_k),
                                       _ptr(param_flat), _stream(stream)), "lags_apply_sparse")

    def lags_delta_monitor(self, table, residual_flat, res_stride, idx, val, P, stride_k, out3, stream=None):
        _check(lib().lags_delta_monitor(self.handle, table.handle, _ptr(residual_flat), int(res_stride), _ptr(idx),
                                        _ptr(val), int(P), int(stride_k), _ptr(out3), _stream(stream)),
               "lags_delta_monitor")

    def lags_last_routes(self, table):
        """Route code per layer of the last lags_sparsify_model call with `table` (diagnostic)."""
        arr = (ctypes.c_int32 * table.n)()
        _check(lib().lags_last_routes(self.handle, table.handle, arr, table.n), "lags_last_routes")
        return list(arr)

    def lags_debug_fallback_chain(self, mode):
        _check(lib().lags_debug_fallback_chain(self.handle, int(mode)), "lags_debug_fallback_chain")

    def lags_debug_scratch_info(self, which):
        """(address, bytes, number of retired buffers) of scratch buffer `which`."""
        p, b, r = ctypes.c_void_p(0), ctypes.c_int64(0), ctypes.c_int64(0)
        _check(lib().lags_debug_scratch_info(self.handle, int(which), ctypes.byref(p), ctypes.byref(b),
                                             ctypes.byref(r)), "lags_debug_scratch_info")
        return (p.value or 0), b.value, r.value

    def lags_debug_poison_scratch(self, stream=None):
        _check(lib().lags_debug_poison_scratch(self.handle, _stream(stream)), "lags_debug_poison_scratch")

    def lags_profile_enable(self, on):
        _check(lib().lags_profile_enable(self.handle, int(bool(on))), "lags_profile_enable")

    def lags_profile_enable_kernel(self, name):
        for kid in range(lib().lags_profile_num_kernels()):
            if lib().lags_profile_kernel_name(kid).decode() == name:
                _check(lib().lags_profile_enable_kernel(self.handle, kid), "lags_profile_enable_kernel")
                return
        raise KeyError(name)

    def lags_profile_reset(self):
        _check(lib().lags_profile_reset(self.handle), "lags_profile_reset")

    def lags_profile_read(self):
        """{kernel name: (total milliseconds, launches)} of everything recorded since the last reset."""
        out = {}
        for kid in range(lib().lags_profile_num_kernels()):
            ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
            _check(lib().lags_profile_read(self.handle, kid, ctypes.byref(ms), ctypes.byref(n)), "lags_profile_read")
            if n.value:
                out[lib().lags_profile_kernel_name(kid).decode()] = (ms.value, n.value)
        return out

    def destroy(self):
        if self.handle:
            lib().lags_destroy(self.handle)
            self.handle = None
