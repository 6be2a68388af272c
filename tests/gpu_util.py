"""Helpers of the GPU parity tests: run the HIP library through its binding on host
arrays, run the oracle on the same bytes, compare bit for bit."""
import concurrent.futures as cf
import os

import numpy as np


def bits(a):
    return np.ascontiguousarray(a, np.float32).view(np.uint32)


def note(msg):
    """Name the case before the GPU step so that a fault can be attributed."""
    print("[gpu-case] " + msg, flush=True)


class Gpu:
    """One library context on cuda:0 plus the torch plumbing."""

    def __init__(self):
        import torch
        from paper_1911_08727_amd import lags
        self.torch = torch
        self.lags = lags
        self.dev = torch.device("cuda:0")
        self.ctx = lags.Context(0)

    def close(self):
        self.ctx.destroy()

    def to_dev(self, a):
        return self.torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)

    def sparsify_model(self, layers, grad, residual, lr, table=None):
        """Host arrays in, host arrays out: (idx, val, new_residual)."""
        t = self.torch
        own = table is None
        if own:
            table = self.ctx.table(layers)
        g, r = self.to_dev(grad), self.to_dev(residual)
        n = table.total_k
        oi = t.full((n,), -7, dtype=t.int32, device=self.dev)
        ov = t.full((n,), float("nan"), dtype=t.float32, device=self.dev)
        self.ctx.lags_sparsify_model(table, g, r, lr, oi, ov)
        t.cuda.synchronize()
        if own:
            table.destroy()
        return oi.cpu().numpy(), ov.cpu().numpy(), r.cpu().numpy()

    def sparsify_layer(self, grad, residual, lr, k):
        t = self.torch
        g, r = self.to_dev(grad), self.to_dev(residual)
        oi = t.full((k,), -7, dtype=t.int32, device=self.dev)
        ov = t.full((k,), float("nan"), dtype=t.float32, device=self.dev)
        self.ctx.lags_sparsify_layer(g, r, lr, k, oi, ov)
        t.cuda.synchronize()
        return oi.cpu().numpy(), ov.cpu().numpy(), r.cpu().numpy()

    def merge(self, layers, idx, val, P, stride_k, total, table=None, fill=123.0):
        t = self.torch
        own = table is None
        if own:
            table = self.ctx.table(layers)
        u = t.full((total,), fill, dtype=t.float32, device=self.dev)
        self.ctx.lags_merge_sparse(table, self.to_dev(idx), self.to_dev(val), P, stride_k, u)
        t.cuda.synchronize()
        if own:
            table.destroy()
        return u.cpu().numpy()


    def apply(self, layers, idx, val, P, stride_k, param, table=None):
        """Host arrays in, the updated parameters out (the input array is not modified)."""
        t = self.torch
        own = table is None
        if own:
            table = self.ctx.table(layers)
        v = self.to_dev(param)
        self.ctx.lags_apply_sparse(table, self.to_dev(idx), self.to_dev(val), P, stride_k, v)
        t.cuda.synchronize()
        if own:
            table.destroy()
        return v.cpu().numpy()

    def delta(self, layers, residual, res_stride, idx, val, P, stride_k, table=None):
        t = self.torch
        own = table is None
        if own:
            table = self.ctx.table(layers)
        out = t.full((len(layers) * 3,), -1.0, dtype=t.float64, device=self.dev)
        self.ctx.lags_delta_monitor(table, self.to_dev(residual), res_stride, self.to_dev(idx), self.to_dev(val),
                                    P, stride_k, out)
        t.cuda.synchronize()
        if own:
            table.destroy()
        return out.cpu().numpy().reshape(len(layers), 3)


def assert_delta_close(name, got, want, rtol=1e-10):
    """Tolerance of the delta metric: both sides sum in double, in the same order over workers;
    only the order of the final sum over elements differs (relative error ~1e-15 * sqrt(d))."""
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape, name
    nan_g, nan_w = np.isnan(got), np.isnan(want)
    assert np.array_equal(nan_g, nan_w), (name, "NaN pattern differs")
    ok = np.isclose(got[~nan_g], want[~nan_w], rtol=rtol, atol=0.0)
    assert ok.all(), (name, got[~nan_g][~ok][:5], want[~nan_w][~ok][:5])


def oracle_model_parallel(oracle, layers, grad, residual, lr, threads=None):
    """The oracle's per-layer function over all layers of a table, layers spread over host
    threads (ctypes releases the GIL).  Same result as oracle.sparsify_model."""
    threads = threads or min(16, os.cpu_count() or 1)
    ks = [oracle.topk_count(d, rho) for (_, d, rho) in layers]
    pos = np.concatenate([[0], np.cumsum(ks)]).astype(np.int64)
    idx = np.empty(pos[-1], np.int32)
    val = np.empty(pos[-1], np.float32)

    def one(l):
        off, d, _ = layers[l]
        i, v = oracle.sparsify_layer(np.ascontiguousarray(grad[off:off + d]), residual[off:off + d], lr, ks[l])
        idx[pos[l]:pos[l + 1]] = i
        val[pos[l]:pos[l + 1]] = v

    order = sorted(range(len(layers)), key=lambda l: -layers[l][1])
    with cf.ThreadPoolExecutor(threads) as ex:
        list(ex.map(one, order))
    return idx, val


def assert_same(name, got, want):
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape, (name, got.shape, want.shape)
    if got.dtype == np.float32:
        got, want = bits(got), bits(want)
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        raise AssertionError("%s: %d of %d differ, first at %d: got %r want %r"
                             % (name, len(bad), got.size, bad[0], got[bad[0]], want[bad[0]]))
