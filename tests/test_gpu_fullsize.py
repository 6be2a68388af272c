"""Full-size GPU checks of benchmark configurations 3, 4 and 5 in the launch configuration
bench.py times: one batched table of P x L layers, one lags_sparsify_model call and one
lags_merge_sparse call per iteration, all P workers, the full iteration count, gradients
generated in device memory.

Every iteration checks, on everything:
  * the merged update against the oracle's merge, bit for bit (all layers);
  * properties that hold at any size, evaluated with torch on the device: exactly k strictly
    ascending in-range indices per layer, values are acc bit for bit, residual is +0 at the
    kept entries and acc elsewhere, every kept magnitude >= every dropped magnitude, and among
    magnitudes equal to the threshold the kept ones have the lowest indices;
and the oracle's sparsifier on the same bytes, bit for bit: on one rotating worker per iteration
and, on the last iteration, on all P workers (every layer of up to 20 M elements; the 103 M-element
layer on one worker).  grad is compared with a copy taken before the call: it is never written.
"""
import numpy as np
import pytest

from gpu_util import assert_delta_close, assert_same, note, oracle_model_parallel
from paper_1911_08727_amd import workloads

pytestmark = pytest.mark.gpu


def _acc(torch, res_before, grad, lr):
    t = torch.mul(grad, float(np.float32(lr)))      # rounded product ...
    return torch.add(res_before, t)                 # ... then rounded sum (two kernels, no fusion)


def _check_properties(torch, wl, layers, ks, pos, P, total, K, acc, res, idx, val):
    keys_all = acc.view(torch.int32) & 0x7FFFFFFF
    for p in range(P):
        for l, (off, d, _) in enumerate(layers):
            k = ks[l]
            i = idx[p * K + pos[l]: p * K + pos[l] + k].long()
            v = val[p * K + pos[l]: p * K + pos[l] + k]
            a = acc[p * total + off: p * total + off + d]
            r = res[p * total + off: p * total + off + d]
            key = keys_all[p * total + off: p * total + off + d]
            assert int(i.min()) >= 0 and int(i.max()) < d
            if k > 1:
                assert bool((i[1:] > i[:-1]).all()), "indices not strictly ascending"
            assert torch.equal(v.view(torch.int32), a[i].view(torch.int32)), "value is not acc"
            mask = torch.zeros(d, dtype=torch.bool, device=a.device)
            mask[i] = True
            assert int(mask.sum()) == k
            assert bool((r[i].view(torch.int32) == 0).all()), "residual not +0 at kept entries"
            assert torch.equal(r.view(torch.int32)[~mask], a.view(torch.int32)[~mask]), "residual is not acc"
            if k < d:
                ksel = key[i]
                T = int(ksel.min())
                dropped = key.masked_fill(mask, -1)
                assert int(dropped.max()) <= T, "a dropped magnitude exceeds a kept one"
                ties_kept = i[ksel == T]
                ties_dropped = torch.nonzero(dropped == T).flatten()
                if len(ties_dropped):
                    assert int(ties_kept.max()) < int(ties_dropped.min()), "tie rule violated"


def _oracle_pairs(oracle, pairs, layers, ks, pos, lr, total, K, grad, res_before, res, hi, hv, it):
    """oracle.sparsify_layer on the listed (worker, layer) pairs, spread over the host threads,
    against the library's pairs and residual, bit for bit."""
    import concurrent.futures as cf
    import os
    host = {}
    for p in sorted(set(p for p, _ in pairs)):
        host[p] = (grad[p * total:(p + 1) * total].cpu().numpy(), res_before[p * total:(p + 1) * total].cpu().numpy(),
                   res[p * total:(p + 1) * total].cpu().numpy())

    def one(pl):
        p, l = pl
        off, d, _ = layers[l]
        g_h, r_h, got_r = host[p]
        r = np.ascontiguousarray(r_h[off:off + d])
        wi, wv = oracle.sparsify_layer(np.ascontiguousarray(g_h[off:off + d]), r, lr, ks[l])
        tag = "it=%d p=%d l=%d" % (it, p, l)
        assert_same("idx " + tag, hi[p * K + pos[l]: p * K + pos[l] + ks[l]], wi)
        assert_same("val " + tag, hv[p * K + pos[l]: p * K + pos[l] + ks[l]], wv)
        assert_same("res " + tag, got_r[off:off + d], r)
        return True

    order = sorted(pairs, key=lambda pl: -layers[pl[1]][1])
    with cf.ThreadPoolExecutor(min(16, os.cpu_count() or 1)) as ex:
        assert all(ex.map(one, order))


def _run_full(name, big_once=(), rho_override=None, iters=None):
    import torch
    import oracle
    from paper_1911_08727_amd import lags
    wl = workloads.make(name, rho_override=rho_override)
    n_iters = iters or wl.iters
    dev = torch.device("cuda:0")
    P, total, layers = wl.P, wl.total_d, wl.layers()
    batched = [(p * total + off, d, r) for p in range(P) for (off, d, r) in layers]
    ctx = lags.Context(0)
    tb, t1 = ctx.table(batched), ctx.table(layers)
    K = t1.total_k
    ks = [t1.k(l) for l in range(len(layers))]
    pos = [t1.out_offset(l) for l in range(len(layers))]
    assert ks == [oracle.topk_count(d, r) for (_, d, r) in layers]
    grad = torch.empty(P * total, dtype=torch.float32, device=dev)
    res = torch.zeros(P * total, dtype=torch.float32, device=dev)
    idx = torch.empty(P * K, dtype=torch.int32, device=dev)
    val = torch.empty(P * K, dtype=torch.float32, device=dev)
    upd = torch.empty(total, dtype=torch.float32, device=dev)
    param = torch.randn(total, dtype=torch.float32, device=dev, generator=torch.Generator(device=dev).manual_seed(7))
    delta = torch.empty(3 * len(layers), dtype=torch.float64, device=dev)
    fell_back = 0
    for it in range(n_iters):
        note("%s iteration %d: generate" % (name, it))
        for p in range(P):
            workloads.grad_torch(wl, it, p, dev, out=grad[p * total:(p + 1) * total])
        res_before = res.clone()
        grad_before = grad.clone()
        note("%s iteration %d: sparsify + merge" % (name, it))
        ctx.lags_sparsify_model(tb, grad, res, wl.lr, idx, val)
        ctx.lags_merge_sparse(t1, idx, val, P, K, upd)
        torch.cuda.synchronize()
        routes = ctx.lags_last_routes(tb)
        fell_back += sum(1 for r in routes if r == 2)

        note("%s iteration %d: merge vs oracle" % (name, it))
        hi, hv = idx.cpu().numpy(), val.cpu().numpy()
        want_u = np.empty(total, np.float32)
        oracle.merge_sparse(layers, hi, hv, P, K, want_u)
        assert_same("update it=%d" % it, upd.cpu().numpy(), want_u)

        note("%s iteration %d: sparse apply vs oracle" % (name, it))
        want_v = param.cpu().numpy()
        oracle.apply_sparse(layers, hi, hv, P, K, want_v)
        ctx.lags_apply_sparse(t1, idx, val, P, K, param)
        torch.cuda.synchronize()
        assert_same("param it=%d" % it, param.cpu().numpy(), want_v)

        if it == n_iters - 1:
            note("%s iteration %d: delta metric vs oracle" % (name, it))
            ctx.lags_delta_monitor(t1, res, total, idx, val, P, K, delta)
            torch.cuda.synchronize()
            want_d = oracle.delta_monitor(layers, res.cpu().numpy(), total, hi, hv, P, K)
            assert_delta_close("delta", delta.cpu().numpy().reshape(-1, 3), want_d)
            # the paper reports delta < 1 on real gradients (Fig. 2); on independent synthetic noise
            # tiny layers (k = 1) scatter around 1, so this is reported, not asserted
            note("%s delta: median %.4f, max %.4f" % (name, np.nanmedian(want_d[:, 2]), np.nanmax(want_d[:, 2])))

        note("%s iteration %d: properties" % (name, it))
        acc = _acc(torch, res_before, grad, wl.lr)
        _check_properties(torch, wl, layers, ks, pos, P, total, K, acc, res, idx, val)
        del acc

        # the oracle's sparsifier on the same bytes: one rotating worker per iteration, and on
        # the last iteration every worker (layers of up to 20 M elements; larger ones where listed
        # in big_once, on the rotating worker only)
        last = it == n_iters - 1
        p_rot = (it * 5 + 3) % P
        workers = list(range(P)) if last else [p_rot]
        small = [l for l, (_, d, _) in enumerate(layers) if d <= 20_000_000]
        pairs = [(p, l) for p in workers for l in small]
        pairs += [(p_rot, l) for l in big_once if last and l not in small]
        note("%s iteration %d: oracle on %d (worker, layer) pairs" % (name, it, len(pairs)))
        _oracle_pairs(oracle, pairs, layers, ks, pos, wl.lr, total, K, grad, res_before, res, hi, hv, it)
        assert torch.equal(grad.view(torch.int32), grad_before.view(torch.int32)), "grad was written"
        del res_before, grad_before
    tb.destroy()
    t1.destroy()
    ctx.destroy()
    return fell_back


def test_vgg16_full():
    """Configuration 3: 32 tensors, 138,357,544 elements, Laplace gradients, rho_l drawn in
    [0.001, 0.01], P = 16, 5 iterations.  fc1 (102.8M elements) goes through the oracle once."""
    fell_back = _run_full("vgg16", big_once=(26,))
    assert fell_back == 0, "a sampled layer fell back to the multi-pass route on smooth data"


def test_vgg16_at_the_benchmarked_density():
    """The workload bench.py times by default: the VGG-16-shaped table with rho = 0.001 for every
    layer, P = 16 in one batched table (nine streaming launches), two iterations."""
    assert _run_full("vgg16", rho_override=0.001, iters=2) == 0


def test_resnet50_full():
    """Configuration 4: 161 tensors, 25,557,032 elements, P = 16, 10 iterations."""
    assert _run_full("resnet50") == 0


def test_lstm_full():
    """Configuration 5: 7 tensors, 66,022,000 elements, embedding gradient non-zero on 2000 of
    10000 rows, rho = 0.005, P = 16, 10 iterations."""
    _run_full("lstm")


def test_inception4_full():
    """The Inception-v4-shaped table (third model of the paper's evaluation): 449 tensors,
    42,679,816 elements, rho = 0.001, P = 16, 3 iterations."""
    assert _run_full("inception4", iters=3) == 0
