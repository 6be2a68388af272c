"""GPU tests at the limits of the interface: the largest layer the ABI admits, resuming from a
saved residual in a fresh context, a non-default stream, the worker-count limit of the merge,
and rejected arguments of the merge-type entry points."""
import numpy as np
import pytest

from gpu_util import Gpu, assert_delta_close, assert_same, note, oracle_model_parallel
from paper_1911_08727_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    g = Gpu()
    yield g
    g.close()


def test_largest_layer_properties(gpu):
    """d = 2^31 - 1 (the largest layer the ABI admits; int32 indices reach 2^31 - 2), checked by
    properties that hold at any size: k strictly ascending in-range indices, values are acc,
    residual is +0 at kept entries and acc elsewhere, kept magnitudes dominate, tie rule."""
    torch = gpu.torch
    d = 2 ** 31 - 1
    k = 2_147_484                          # ceil(0.001 * d)
    gen = torch.Generator(device=gpu.dev).manual_seed(5)
    g = torch.empty(d, dtype=torch.float32, device=gpu.dev)
    g.normal_(0.0, 1.0, generator=gen)
    g[-1] = 100.0                          # the last element must be kept: index 2^31 - 2
    res0 = torch.empty(d, dtype=torch.float32, device=gpu.dev)
    res0.normal_(0.0, 0.5, generator=gen)
    res = res0.clone()
    oi = torch.empty(k, dtype=torch.int32, device=gpu.dev)
    ov = torch.empty(k, dtype=torch.float32, device=gpu.dev)
    note("largest layer d=%d k=%d" % (d, k))
    gpu.ctx.lags_sparsify_layer(g, res, 0.1, k, oi, ov)
    torch.cuda.synchronize()
    acc = torch.add(res0, torch.mul(g, float(np.float32(0.1))))
    del g, res0
    i = oi.long()
    assert int(i[0]) >= 0 and int(i[-1]) == d - 1
    assert bool((i[1:] > i[:-1]).all())
    assert torch.equal(ov.view(torch.int32), acc[i].view(torch.int32))
    assert bool((res[i].view(torch.int32) == 0).all())
    key = acc.view(torch.int32) & 0x7FFFFFFF
    T = int(key[i].min())
    ties_kept = i[key[i] == T]
    res_bits = res.view(torch.int32)
    acc_bits = acc.view(torch.int32)
    acc_bits[i] = 0                        # acc with the kept entries zeroed is the expected residual
    assert torch.equal(res_bits, acc_bits)
    key[i] = -1
    assert int(key.max()) <= T
    dropped_ties = torch.nonzero(key == T).flatten()
    if len(dropped_ties):
        assert int(ties_kept.max()) < int(dropped_ties.min())


def test_resume_from_saved_residual(gpu, oracle):
    """The context holds nothing that influences results: 6 iterations in one context equal
    3 iterations, a fresh context fed the saved residual, and 3 more."""
    from paper_1911_08727_amd import lags
    rng = np.random.default_rng(71)
    layers = [(0, 200_000, 0.002), (200_000, 5_000, 0.01), (205_000, 90_000, 0.001)]
    total = 295_000
    grads = [rng.standard_normal(total).astype(np.float32) for _ in range(6)]
    straight = np.zeros(total, np.float32)
    outs = []
    for it in range(6):
        note("resume: straight iteration %d" % it)
        gi, gv, straight = gpu.sparsify_model(layers, grads[it], straight, 0.1)
        outs.append((gi, gv))
    res = np.zeros(total, np.float32)
    for it in range(3):
        _, _, res = gpu.sparsify_model(layers, grads[it], res, 0.1)
    other = Gpu()
    try:
        for it in range(3, 6):
            note("resume: fresh context iteration %d" % it)
            gi, gv, res = other.sparsify_model(layers, grads[it], res, 0.1)
            assert_same("idx it=%d" % it, gi, outs[it][0])
            assert_same("val it=%d" % it, gv, outs[it][1])
    finally:
        other.close()
    assert_same("residual", res, straight)


def test_non_default_stream(gpu, oracle):
    """Work is enqueued on the stream the caller names and ordered with the caller's other work on it."""
    torch = gpu.torch
    rng = np.random.default_rng(73)
    layers = [(0, 500_000, 0.001), (500_000, 3000, 0.01)]
    total = 503_000
    g_h = rng.standard_normal(total).astype(np.float32)
    want_r = np.zeros(total, np.float32)
    wi, wv = oracle_model_parallel(oracle, layers, g_h, want_r, 0.1)
    table = gpu.ctx.table(layers)
    K = table.total_k
    stream = torch.cuda.Stream(device=gpu.dev)          # default priority
    g = gpu.to_dev(g_h)
    oi = torch.empty(K, dtype=torch.int32, device=gpu.dev)
    ov = torch.empty(K, dtype=torch.float32, device=gpu.dev)
    upd = torch.empty(total, dtype=torch.float32, device=gpu.dev)
    torch.cuda.synchronize()
    note("non-default stream")
    with torch.cuda.stream(stream):
        r = torch.zeros(total, dtype=torch.float32, device=gpu.dev)   # produced on the same stream
        gpu.ctx.lags_sparsify_model(table, g, r, 0.1, oi, ov, stream)
        gpu.ctx.lags_merge_sparse(table, oi, ov, 1, K, upd, stream)
    stream.synchronize()
    assert_same("idx", oi.cpu().numpy(), wi)
    assert_same("val", ov.cpu().numpy(), wv)
    assert_same("res", r.cpu().numpy(), want_r)
    want_u = np.empty(total, np.float32)
    oracle.merge_sparse(layers, wi, wv, 1, K, want_u)
    assert_same("update", upd.cpu().numpy(), want_u)
    table.destroy()


def test_merge_worker_limit_and_rejected_arguments(gpu, oracle):
    """P = 1024 is the most the merge accepts; P = 0, P = 1025, a pair stride below sum k, a
    worker stride below the model and null pointers are rejected before anything is written."""
    torch = gpu.torch
    from paper_1911_08727_amd import lags
    rng = np.random.default_rng(79)
    layers = [(0, 3000, 0.002), (3000, 9000, 0.001)]
    total, K, P = 12000, oracle.total_k(layers), 1024
    idx = np.empty(P * K, np.int32)
    val = rng.standard_normal(P * K).astype(np.float32)
    for p in range(P):
        pos = 0
        for (_, d, rho) in layers:
            k = oracle.topk_count(d, rho)
            idx[p * K + pos:p * K + pos + k] = np.sort(rng.choice(d, k, replace=False))
            pos += k
    note("merge with P=1024")
    want = np.empty(total, np.float32)
    oracle.merge_sparse(layers, idx, val, P, K, want)
    assert_same("update", gpu.merge(layers, idx, val, P, K, total), want)

    table = gpu.ctx.table(layers)
    di, dv = gpu.to_dev(idx), gpu.to_dev(val)
    upd = torch.full((total,), 5.0, dtype=torch.float32, device=gpu.dev)
    out3 = torch.full((6,), 5.0, dtype=torch.float64, device=gpu.dev)
    res = torch.zeros(2 * total, dtype=torch.float32, device=gpu.dev)
    for bad in (dict(P=0), dict(P=1025), dict(stride=K - 1)):
        with pytest.raises(lags.LagsError):
            gpu.ctx.lags_merge_sparse(table, di, dv, bad.get("P", 2), bad.get("stride", K), upd)
        with pytest.raises(lags.LagsError):
            gpu.ctx.lags_apply_sparse(table, di, dv, bad.get("P", 2), bad.get("stride", K), upd)
        with pytest.raises(lags.LagsError):
            gpu.ctx.lags_delta_monitor(table, res, total, di, dv, bad.get("P", 2), bad.get("stride", K), out3)
    with pytest.raises(lags.LagsError):
        gpu.ctx.lags_delta_monitor(table, res, total - 1, di, dv, 2, K, out3)     # workers would overlap
    with pytest.raises(lags.LagsError):
        gpu.ctx.lags_merge_sparse(table, None, dv, 2, K, upd)
    with pytest.raises(lags.LagsError):
        gpu.ctx.lags_apply_sparse(table, di, dv, 2, K, None)
    torch.cuda.synchronize()
    assert bool((upd == 5.0).all()) and bool((out3 == 5.0).all())
    with pytest.raises(lags.LagsError):
        gpu.ctx.table([])                                                         # no layers
    with pytest.raises(lags.LagsError):
        gpu.ctx.table([(0, 0, 0.5)])                                              # empty layer
    with pytest.raises(lags.LagsError):
        gpu.ctx.table([(0, 2 ** 31, 0.5)])                                        # beyond int32 indices
    table.destroy()


def test_hip_graph_replay_matches_eager_and_oracle(gpu, oracle):
    """One step (batched sparsify of P workers + merge) captured into a HIP graph after a warm-up
    call has sized the scratch; every replay, with eager work and synchronisations of the program
    between the replays, equals the eager calls and the oracle bit for bit.  The capture includes
    the fork to and join from the context's side stream and uses clearing kernels, no memset."""
    torch = gpu.torch
    rng = np.random.default_rng(77)
    sizes = [(100, 0.01), (300_000, 0.002), (60_000, 0.6), (9000, 0.001), (2_200_000, 0.01), (1 << 20, 0.001)]
    layers, off = [], 0
    for d, rho in sizes:
        layers.append((off, d, rho))
        off += d
    total, P, lr = off, 2, 0.1
    batched = [(p * total + o, d, r) for p in range(P) for (o, d, r) in layers]
    tb, t1 = gpu.ctx.table(batched), gpu.ctx.table(layers)
    K = t1.total_k
    g_host = rng.standard_normal(P * total).astype(np.float32)
    r_host = (0.1 * rng.standard_normal(P * total)).astype(np.float32)
    grad, res0 = gpu.to_dev(g_host), gpu.to_dev(r_host)
    res = res0.clone()
    idx = torch.empty(P * K, dtype=torch.int32, device=gpu.dev)
    val = torch.empty(P * K, dtype=torch.float32, device=gpu.dev)
    upd = torch.empty(total, dtype=torch.float32, device=gpu.dev)
    note("graph test: warm-up call outside capture")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        gpu.ctx.lags_sparsify_model(tb, grad, res, lr, idx, val, side)
        gpu.ctx.lags_merge_sparse(t1, idx, val, P, K, upd, side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    res.copy_(res0)
    note("graph test: capture")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        st = torch.cuda.current_stream()
        gpu.ctx.lags_sparsify_model(tb, grad, res, lr, idx, val, st)
        gpu.ctx.lags_merge_sparse(t1, idx, val, P, K, upd, st)
    res_cpu = [r_host[p * total:(p + 1) * total].copy() for p in range(P)]
    for it in range(3):
        note("graph test: replay %d" % it)
        graph.replay()
        torch.cuda.synchronize()
        _ = float((grad * 2.0).sum().item())          # eager work between the replays
        want_i, want_v = np.empty(P * K, np.int32), np.empty(P * K, np.float32)
        for p in range(P):
            wi, wv = oracle_model_parallel(oracle, layers, g_host[p * total:(p + 1) * total], res_cpu[p], lr)
            want_i[p * K:(p + 1) * K], want_v[p * K:(p + 1) * K] = wi, wv
        want_u = np.zeros(total, np.float32)
        oracle.merge_sparse(layers, want_i, want_v, P, K, want_u)
        assert_same("idx replay %d" % it, idx.cpu().numpy(), want_i)
        assert_same("val replay %d" % it, val.cpu().numpy(), want_v)
        assert_same("res replay %d" % it, res.cpu().numpy(), np.concatenate(res_cpu))
        assert_same("update replay %d" % it, upd.cpu().numpy(), want_u)
    del graph
    tb.destroy()
    t1.destroy()


def test_two_contexts_on_two_streams(gpu, oracle):
    """Two contexts, each on a stream of its own, enqueue their steps without waiting for each
    other (a context holds all scratch; nothing is shared between contexts): both results equal
    the oracle."""
    torch = gpu.torch
    from paper_1911_08727_amd import lags
    rng = np.random.default_rng(78)
    sizes = [(500, 0.01), (700_000, 0.002), (50_000, 0.5), (1_500_000, 0.01), (45_000, 0.001)]
    layers, off = [], 0
    for d, rho in sizes:
        layers.append((off, d, rho))
        off += d
    total = off
    ctxs = [gpu.ctx, lags.Context(0)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    tables = [c.table(layers) for c in ctxs]
    K = tables[0].total_k
    g_host = [rng.standard_normal(total).astype(np.float32) for _ in ctxs]
    r_host = [(0.2 * rng.standard_normal(total)).astype(np.float32) for _ in ctxs]
    grad = [gpu.to_dev(g) for g in g_host]
    res = [gpu.to_dev(r) for r in r_host]
    idx = [torch.empty(K, dtype=torch.int32, device=gpu.dev) for _ in ctxs]
    val = [torch.empty(K, dtype=torch.float32, device=gpu.dev) for _ in ctxs]
    upd = [torch.empty(total, dtype=torch.float32, device=gpu.dev) for _ in ctxs]
    torch.cuda.synchronize()
    note("two contexts: enqueue three steps each, interleaved")
    for it in range(3):
        for i in (0, 1):
            with torch.cuda.stream(streams[i]):
                ctxs[i].lags_sparsify_model(tables[i], grad[i], res[i], 0.3, idx[i], val[i], streams[i])
                ctxs[i].lags_merge_sparse(tables[i], idx[i], val[i], 1, K, upd[i], streams[i])
    torch.cuda.synchronize()
    for i in (0, 1):
        rc = r_host[i].copy()
        for it in range(3):
            wi, wv = oracle_model_parallel(oracle, layers, g_host[i], rc, 0.3)
        want_u = np.zeros(total, np.float32)
        oracle.merge_sparse(layers, wi, wv, 1, K, want_u)
        assert_same("idx ctx %d" % i, idx[i].cpu().numpy(), wi)
        assert_same("val ctx %d" % i, val[i].cpu().numpy(), wv)
        assert_same("res ctx %d" % i, res[i].cpu().numpy(), rc)
        assert_same("update ctx %d" % i, upd[i].cpu().numpy(), want_u)
    for t in tables:
        t.destroy()
    ctxs[1].destroy()


def test_context_without_side_stream(gpu, oracle, monkeypatch):
    """LAGS_SIDE_STREAM=0 at lags_create keeps every kernel on the caller's stream: a table with
    small and large layers gives the oracle's results over several iterations."""
    from paper_1911_08727_amd import lags
    torch = gpu.torch
    monkeypatch.setenv("LAGS_SIDE_STREAM", "0")
    ctx = lags.Context(0)
    monkeypatch.delenv("LAGS_SIDE_STREAM")
    rng = np.random.default_rng(79)
    sizes = [(900, 0.01), (6_000, 0.004), (300_000, 0.002), (30_000, 0.001), (2_300_000, 0.001), (70_000, 0.4)]
    layers, off = [], 0
    for d, rho in sizes:
        layers.append((off, d, rho))
        off += d + 1
    table = ctx.table(layers)
    K = table.total_k
    res = torch.zeros(off, dtype=torch.float32, device=gpu.dev)
    idx = torch.empty(K, dtype=torch.int32, device=gpu.dev)
    val = torch.empty(K, dtype=torch.float32, device=gpu.dev)
    rc = np.zeros(off, np.float32)
    stream = torch.cuda.current_stream()
    for it in range(3):
        note("one-stream context, iteration %d" % it)
        g = rng.standard_normal(off).astype(np.float32)
        wi, wv = oracle_model_parallel(oracle, layers, g, rc, 0.2)
        ctx.lags_sparsify_model(table, gpu.to_dev(g), res, 0.2, idx, val, stream)
        torch.cuda.synchronize()
        assert_same("idx", idx.cpu().numpy(), wi)
        assert_same("val", val.cpu().numpy(), wv)
        assert_same("res", res.cpu().numpy(), rc)
    table.destroy()
    ctx.destroy()


def _one_table_case(rng, sizes):
    layers, off = [], 0
    for d, rho in sizes:
        layers.append((off, d, rho))
        off += d
    return layers, off


def test_graph_survives_scratch_growth(oracle):
    """A graph recorded with a small table stays valid after a much larger table made the
    context's scratch grow: outgrown buffers are kept until lags_destroy once a call has been
    recorded (before that they are freed), so the replay still finds its scratch."""
    import torch
    from paper_1911_08727_amd import lags
    g = Gpu()
    try:
        rng = np.random.default_rng(91)
        small_layers, total = _one_table_case(rng, [(300_000, 0.002), (2000, 0.01), (2_300_000, 0.001)])
        tiny = g.ctx.table([(0, 50_000, 0.01)])
        before = g.ctx.lags_debug_scratch_info(5)          # the candidate slots
        ts = g.ctx.table(small_layers)
        after = g.ctx.lags_debug_scratch_info(5)
        assert after[1] > before[1] and after[2] == 0, "growth before any capture frees the old buffer"
        K = ts.total_k
        g_host = rng.standard_normal(total).astype(np.float32)
        r_host = (0.1 * rng.standard_normal(total)).astype(np.float32)
        grad, res0 = g.to_dev(g_host), g.to_dev(r_host)
        res = res0.clone()
        idx = torch.empty(K, dtype=torch.int32, device=g.dev)
        val = torch.empty(K, dtype=torch.float32, device=g.dev)
        note("growth test: warm-up and capture with the small table")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            g.ctx.lags_sparsify_model(ts, grad, res, 0.1, idx, val, side)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        res.copy_(res0)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            g.ctx.lags_sparsify_model(ts, grad, res, 0.1, idx, val, torch.cuda.current_stream())
        note("growth test: a larger table moves the scratch")
        big_layers, big_total = _one_table_case(rng, [(6_000_000, 0.004), (3_000_000, 0.001)])
        tb = g.ctx.table(big_layers)
        grown = g.ctx.lags_debug_scratch_info(5)
        assert grown[0] != after[0] and grown[1] > after[1], "the slots were expected to move"
        assert grown[2] >= 1, "the outgrown buffer must be kept for the recorded graph"
        gb = torch.randn(big_total, device=g.dev)
        rb = torch.zeros(big_total, device=g.dev)
        ib = torch.empty(tb.total_k, dtype=torch.int32, device=g.dev)
        vb = torch.empty(tb.total_k, dtype=torch.float32, device=g.dev)
        g.ctx.lags_sparsify_model(tb, gb, rb, 0.1, ib, vb)
        torch.cuda.synchronize()
        res_cpu = r_host.copy()
        for it in range(2):
            note("growth test: replay %d of the graph recorded before the growth" % it)
            graph.replay()
            torch.cuda.synchronize()
            wi, wv = oracle_model_parallel(oracle, small_layers, g_host, res_cpu, 0.1)
            assert_same("idx replay %d" % it, idx.cpu().numpy(), wi)
            assert_same("val replay %d" % it, val.cpu().numpy(), wv)
            assert_same("res replay %d" % it, res.cpu().numpy(), res_cpu)
        del graph
        for t in (tiny, ts, tb):
            t.destroy()
    finally:
        g.close()


def test_scratch_poison_does_not_change_results(gpu, oracle):
    """Scratch carries nothing between calls: with every scratch buffer of the context overwritten
    by 0xFF bytes before the call, a table whose layers take all routes (one-workgroup, sampled
    with one and with many workgroups, rejected guess, multi-pass) gives the oracle's bits, and so
    do the merge, the apply and the delta metric."""
    torch = gpu.torch
    rng = np.random.default_rng(92)
    sizes = [(700, 0.01), (250_000, 0.002), (2_600_000, 0.003), (60_000, 0.6), (180_000, 0.001), (7_000, 0.004)]
    layers, total = _one_table_case(rng, sizes)
    P = 3
    table = gpu.ctx.table(layers)
    K = table.total_k
    g_host = [rng.standard_normal(total).astype(np.float32) for _ in range(P)]
    for gh in g_host:
        o, d, _ = layers[4]
        gh[o:o + d] = 0.0                                   # an all-zero layer: the guess is rejected
    r_host = [(0.2 * rng.standard_normal(total)).astype(np.float32) for _ in range(P)]
    for rh in r_host:
        o, d, _ = layers[4]
        rh[o:o + d] = 0.0
    for mode in (0, 1, 2, 0):
        gpu.ctx.lags_debug_fallback_chain(mode)
        res_cpu = [r.copy() for r in r_host]
        all_i, all_v = np.empty(P * K, np.int32), np.empty(P * K, np.float32)
        res_dev = torch.empty(P * total, dtype=torch.float32, device=gpu.dev)
        for p in range(P):
            note("poison test: fallback mode %d, worker %d" % (mode, p))
            gpu.ctx.lags_debug_poison_scratch()
            wi, wv = oracle_model_parallel(oracle, layers, g_host[p], res_cpu[p], 0.5)
            gi, gv, gr = gpu.sparsify_model(layers, g_host[p], r_host[p], 0.5, table=table)
            routes = gpu.ctx.lags_last_routes(table)
            assert routes == [0, 1, 1, 3, 2, 0], routes
            assert_same("idx", gi, wi)
            assert_same("val", gv, wv)
            assert_same("res", gr, res_cpu[p])
            all_i[p * K:(p + 1) * K], all_v[p * K:(p + 1) * K] = gi, gv
            res_dev[p * total:(p + 1) * total] = gpu.to_dev(gr)
        note("poison test: merge, apply, delta after poisoning")
        want_u = np.full(total, 5.0, np.float32)
        oracle.merge_sparse(layers, all_i, all_v, P, K, want_u)
        gpu.ctx.lags_debug_poison_scratch()
        assert_same("update", gpu.merge(layers, all_i, all_v, P, K, total, table=table, fill=5.0), want_u)
        param = rng.standard_normal(total).astype(np.float32)
        want_v = param.copy()
        oracle.apply_sparse(layers, all_i, all_v, P, K, want_v)
        gpu.ctx.lags_debug_poison_scratch()
        assert_same("param", gpu.apply(layers, all_i, all_v, P, K, param, table=table), want_v)
        gpu.ctx.lags_debug_poison_scratch()
        got_d = gpu.delta(layers, res_dev.cpu().numpy(), total, all_i, all_v, P, K, table=table)
        want_d = oracle.delta_monitor(layers, res_dev.cpu().numpy(), total, all_i, all_v, P, K)
        assert_delta_close("delta", got_d, want_d)
    gpu.ctx.lags_debug_fallback_chain(0)
    table.destroy()


def test_rejected_guesses_on_layers_finished_by_groups(gpu, oracle):
    """Layers of more than 512 tiles (finished by groups of workgroups) whose guess is rejected,
    served by the one-workgroup selection (mode 2), by the multi-pass kernels (mode 1) and in the
    default mode: an all-zero layer (rejected when the candidates are counted), a layer with 300
    entries tied at the k-th largest magnitude inside one group (that group's share of the band
    overflows: rejected between the group phases), the same ties spread over the layer (accepted)."""
    rng = np.random.default_rng(93)
    d, rho = 2_400_000, 0.001
    k = 2400
    base = rng.standard_normal(d).astype(np.float32)
    mags = np.sort(np.abs(base))[::-1]
    v = np.float32(mags[k - 150])                     # 300 ties at v straddle rank k
    tied_one_group = base.copy()
    tied_one_group[786_432 + np.arange(300) * 800] = v   # inside one group of 64 tiles, a few per tile
    tied_spread = base.copy()
    tied_spread[np.arange(300) * 7919 + 5] = -v
    cases = [("zeros", np.zeros(d, np.float32), 2), ("ties in one group", tied_one_group, 2),
             ("ties spread", tied_spread, 1)]
    for mode in (2, 1, 0):
        gpu.ctx.lags_debug_fallback_chain(mode)
        for name, g, want_route in cases:
            note("group rejection: mode %d, %s" % (mode, name))
            routes = _check(gpu, oracle, [(0, d, rho)], g, np.zeros(d, np.float32), 1.0)
            assert routes == [want_route], (name, mode, routes)
    gpu.ctx.lags_debug_fallback_chain(0)


def _check(gpu, oracle, layers, g, r0, lr):
    table = gpu.ctx.table(layers)
    want_r = r0.copy()
    wi, wv = oracle_model_parallel(oracle, layers, g, want_r, lr)
    gi, gv, gr = gpu.sparsify_model(layers, g, r0, lr, table=table)
    routes = gpu.ctx.lags_last_routes(table)
    table.destroy()
    assert_same("idx", gi, wi)
    assert_same("val", gv, wv)
    assert_same("res", gr, want_r)
    return routes
