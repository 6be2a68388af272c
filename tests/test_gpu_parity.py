"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, bit for bit,
on the same seeded inputs.  Bar: indices, values, residuals and the merged update are
integer/bit identical (the arithmetic is two binary32 roundings on both sides; where a
float decides the selection both sides decide on the same binary32 acc bits)."""
import zlib

import numpy as np
import pytest

from gpu_util import Gpu, assert_delta_close, assert_same, bits, note, oracle_model_parallel
from paper_1911_08727_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    g = Gpu()
    yield g
    g.close()


def _values(kind, d, rng):
    if kind == "normal":
        return rng.standard_normal(d).astype(np.float32)
    if kind == "ties":
        return rng.integers(-3, 4, d).astype(np.float32)
    if kind == "zeros":
        return np.zeros(d, np.float32)
    if kind == "equal":
        return np.full(d, -2.5, np.float32)
    if kind == "signed_zeros":
        return np.where(rng.random(d) < 0.5, np.float32(0.0), np.float32(-0.0)).astype(np.float32)
    if kind == "denormal":
        return (rng.integers(-50, 51, d).astype(np.float64) * 2.0 ** -149).astype(np.float32)
    if kind == "mostly_zero":
        x = rng.standard_normal(d).astype(np.float32)
        x[rng.random(d) < 0.9] = 0.0
        return x
    if kind == "narrow":          # all magnitudes inside one top-level radix bin
        return (1.0 + rng.random(d) * 0.01).astype(np.float32) * rng.choice([-1, 1], d).astype(np.float32)
    if kind == "inf":
        x = rng.standard_normal(d).astype(np.float32)
        x[rng.integers(0, d, max(1, d // 50))] = np.inf
        x[rng.integers(0, d, max(1, d // 50))] = -np.inf
        return x
    raise KeyError(kind)


KINDS = ["normal", "ties", "zeros", "equal", "signed_zeros", "denormal", "mostly_zero", "narrow", "inf"]
# sizes around every boundary of the launch plan: vector width, wave, small classes, tile
SIZES = [1, 2, 3, 4, 5, 63, 64, 65, 255, 256, 257, 1023, 1024, 1025, 4100, 8191, 8192, 8193,
         40959, 40960, 40961, 45055, 45056, 45057, 3 * 8192, 3 * 8192 + 5, 100003]


def _ks(d, rng):
    ks = {1, d, max(1, d // 2), max(1, int(np.ceil(0.001 * d))), max(1, int(np.ceil(0.01 * d)))}
    if d > 3:
        ks.add(int(rng.integers(2, d)))
    return sorted(ks)


@pytest.mark.parametrize("kind", KINDS)
def test_single_layer_edges(gpu, oracle, kind):
    """lags_sparsify_layer on crafted layers at every size boundary and several k."""
    rng = np.random.default_rng(zlib.crc32(kind.encode()))
    lr = np.float32(0.3)
    for d in SIZES:
        g = _values(kind, d, rng)
        r0 = (_values(kind, d, rng) * np.float32(0.5)).astype(np.float32)
        if kind == "inf":
            r0[~np.isfinite(r0)] = 1.0          # keep acc free of inf - inf
            r0[~np.isfinite(g)] = 0.0
        for k in _ks(d, rng):
            note("edges kind=%s d=%d k=%d" % (kind, d, k))
            want_r = r0.copy()
            wi, wv = oracle.sparsify_layer(g, want_r, lr, k)
            gi, gv, gr = gpu.sparsify_layer(g, r0, lr, k)
            assert_same("idx %s d=%d k=%d" % (kind, d, k), gi, wi)
            assert_same("val %s d=%d k=%d" % (kind, d, k), gv, wv)
            assert_same("res %s d=%d k=%d" % (kind, d, k), gr, want_r)


def test_fma_would_differ(gpu, oracle):
    """The accumulate is a rounded product then a rounded sum: inputs where a fused
    multiply-add gives other bits (and another selection) must match the oracle."""
    d = 5000
    rng = np.random.default_rng(3)
    g = rng.standard_normal(d).astype(np.float32)
    r0 = (-np.float32(0.1) * g).astype(np.float32)      # acc is exactly the product's rounding error...
    r0[::7] += np.float32(1e-9)
    g[0], r0[0] = 3.0, -0.3                              # the hand-worked element: acc == +0.0
    want_r = r0.copy()
    wi, wv = oracle.sparsify_layer(g, want_r, np.float32(0.1), 40)
    gi, gv, gr = gpu.sparsify_layer(g, r0, np.float32(0.1), 40)
    assert bits(gr)[0] == 0
    assert_same("idx", gi, wi)
    assert_same("val", gv, wv)
    assert_same("res", gr, want_r)


def test_unaligned_offsets_and_gaps(gpu, oracle):
    """Layers at arbitrary element offsets (not multiples of 4), with gaps between them."""
    rng = np.random.default_rng(8)
    sizes = [7, 1, 300, 1025, 9000, 41001, 70001, 13]
    layers, off = [], 3
    for d in sizes:
        layers.append((off, d, float(rng.choice([0.001, 0.01, 0.3, 1.0]))))
        off += d + int(rng.integers(0, 6))
    total = off + 5
    g = rng.standard_normal(total).astype(np.float32)
    r0 = rng.standard_normal(total).astype(np.float32)
    note("unaligned offsets")
    want_r = r0.copy()
    wi, wv = oracle.sparsify_model(layers, g, want_r, 0.05)
    gi, gv, gr = gpu.sparsify_model(layers, g, r0, 0.05)
    assert_same("idx", gi, wi)
    assert_same("val", gv, wv)
    assert_same("res", gr, want_r)            # includes the untouched gaps


def test_nan_inputs_select_same_indices(gpu, oracle):
    """NaN keys rank above infinity on both sides; NaN payloads are not compared."""
    d = 3000
    rng = np.random.default_rng(12)
    g = rng.standard_normal(d).astype(np.float32)
    g[[5, 77, 2048]] = np.nan
    r0 = np.zeros(d, np.float32)
    want_r = r0.copy()
    wi, _ = oracle.sparsify_layer(g, want_r, 1.0, 10)
    gi, gv, gr = gpu.sparsify_layer(g, r0, 1.0, 10)
    assert_same("idx", gi, wi)
    assert np.isnan(gv[np.isin(gi, [5, 77, 2048])]).all()
    assert_same("res", gr, want_r)


def _run_config(gpu, oracle, wl, iters, P, check_merge=True):
    layers = wl.layers()
    total = wl.total_d
    table = gpu.ctx.table(layers)
    K = table.total_k
    assert K == oracle.total_k(layers)
    res_gpu = [np.zeros(total, np.float32) for _ in range(P)]
    res_cpu = [np.zeros(total, np.float32) for _ in range(P)]
    for it in range(iters):
        all_i = np.empty(P * K, np.int32)
        all_v = np.empty(P * K, np.float32)
        for p in range(P):
            note("config %s iteration %d worker %d" % (wl.name, it, p))
            g = workloads.grad_numpy(wl, it, p)
            gi, gv, gr = gpu.sparsify_model(layers, g, res_gpu[p], wl.lr, table=table)
            wi, wv = oracle_model_parallel(oracle, layers, g, res_cpu[p], wl.lr)
            assert_same("idx it=%d p=%d" % (it, p), gi, wi)
            assert_same("val it=%d p=%d" % (it, p), gv, wv)
            assert_same("res it=%d p=%d" % (it, p), gr, res_cpu[p])
            res_gpu[p] = gr
            all_i[p * K:(p + 1) * K] = gi
            all_v[p * K:(p + 1) * K] = gv
        if check_merge:
            note("config %s iteration %d merge" % (wl.name, it))
            want_u = np.full(total, 123.0, np.float32)
            oracle.merge_sparse(layers, all_i, all_v, P, K, want_u)
            got_u = gpu.merge(layers, all_i, all_v, P, K, total, table=table)
            assert_same("update it=%d" % it, got_u, want_u)
            note("config %s iteration %d apply" % (wl.name, it))
            param = np.random.default_rng(it).standard_normal(total).astype(np.float32)
            got_v = gpu.apply(layers, all_i, all_v, P, K, param, table=table)
            want_v = param.copy()
            oracle.apply_sparse(layers, all_i, all_v, P, K, want_v)
            assert_same("param it=%d" % it, got_v, want_v)
            assert_same("param = v - update it=%d" % it, got_v, param - want_u)
            note("config %s iteration %d delta" % (wl.name, it))
            res_all = np.concatenate(res_gpu)
            want_d = oracle.delta_monitor(layers, res_all, total, all_i, all_v, P, K)
            got_d = gpu.delta(layers, res_all, total, all_i, all_v, P, K, table=table)
            assert_delta_close("delta it=%d" % it, got_d, want_d)
    table.destroy()


def test_config_single_tensor(gpu, oracle):
    """Benchmark configuration 1 in full: d = 2^20, k = 1049, P = 4, 10 iterations."""
    wl = workloads.make("single")
    _run_config(gpu, oracle, wl, wl.iters, wl.P)


def test_config_resnet20(gpu, oracle):
    """Benchmark configuration 2 in full: 58 tensors, P = 16, 20 iterations."""
    wl = workloads.make("resnet20")
    _run_config(gpu, oracle, wl, wl.iters, wl.P)


def test_config_resnet50_reduced(gpu, oracle):
    """Configuration 4's full table; 2 workers x 3 iterations against the full oracle
    (the full worker and iteration counts run in test_gpu_fullsize.py on sampled layers)."""
    wl = workloads.make("resnet50")
    _run_config(gpu, oracle, wl, 3, 2)


def _check_table(gpu, oracle, layers, g, r0, lr, want_routes=None):
    table = gpu.ctx.table(layers)
    want_r = r0.copy()
    wi, wv = oracle_model_parallel(oracle, layers, g, want_r, lr)
    gi, gv, gr = gpu.sparsify_model(layers, g, r0, lr, table=table)
    routes = gpu.ctx.lags_last_routes(table)
    table.destroy()
    assert_same("idx", gi, wi)
    assert_same("val", gv, wv)
    assert_same("res", gr, want_r)
    if want_routes is not None:
        assert routes == want_routes, routes
    return routes


def test_sampled_route_is_taken_and_exact(gpu, oracle):
    """Large layers with smooth value distributions go through the sampled threshold
    (route 1) with short and with multi-tile candidate lists; results equal the oracle."""
    rng = np.random.default_rng(51)
    sizes = [(1 << 20, 0.001), (3_000_017, 0.01), (70_001, 0.001), (500_000, 0.02), (41_000, 0.005),
             (2_500_000, 0.0004), (600_000, 0.1), (90_000, 0.18)]
    layers, off = [], 0
    for d, rho in sizes:
        layers.append((off, d, rho))
        off += d
    g = rng.standard_normal(off).astype(np.float32)
    g[: 1 << 20] = rng.laplace(size=1 << 20).astype(np.float32)
    r0 = (0.5 * rng.standard_normal(off)).astype(np.float32)
    note("sampled route, smooth data")
    routes = _check_table(gpu, oracle, layers, g, r0, 0.1)
    assert routes == [1] * len(sizes), routes


def test_sampled_route_rejections_fall_back(gpu, oracle):
    """Inputs on which the guessed threshold cannot work (all equal, all zero, few non-zeros,
    heavy ties, a k that is most of the layer) take the exact fallback and match the oracle;
    a layer with clustered large values may overflow single chunks and fall back too."""
    rng = np.random.default_rng(52)
    d = 300_000
    cases = {
        "zeros": np.zeros(d, np.float32),
        "equal": np.full(d, 3.25, np.float32),
        "few_nonzero": np.where(rng.random(d) < 0.0005, rng.standard_normal(d), 0.0).astype(np.float32),
        "narrow": (1.0 + 1e-4 * rng.random(d)).astype(np.float32),
        "ties": rng.integers(-2, 3, d).astype(np.float32),
        "clustered": np.where(np.arange(d) // 3000 % 10 == 0, 50.0, 1.0).astype(np.float32)
                     * rng.standard_normal(d).astype(np.float32),
    }
    for name, g in cases.items():
        for rho in (0.001, 0.01):
            note("rejection case %s rho=%g" % (name, rho))
            routes = _check_table(gpu, oracle, [(0, d, rho)], g, np.zeros(d, np.float32), 1.0)
            assert routes[0] in (1, 2)
            if name in ("zeros", "equal"):
                assert routes == [2], (name, routes)
            if name == "narrow":          # the threshold is a full 31-bit key, so one radix bin is no obstacle
                assert routes == [1], (name, routes)
    note("rejection case large k")
    g = rng.standard_normal(d).astype(np.float32)
    assert _check_table(gpu, oracle, [(0, d, 0.5)], g, np.zeros(d, np.float32), 1.0) == [3]


def test_fallback_after_early_zeros(gpu, oracle):
    """A large layer with k >= 8192 (so the streaming pass zeroes the entries it expects to be
    kept) whose candidates overflow the slots of a few tiles: the layer falls back to the
    multi-pass route, which must first see every early zero undone."""
    rng = np.random.default_rng(54)
    d, rho = 2_000_000, 0.01
    g = rng.standard_normal(d).astype(np.float32)
    g[100_000:110_000] *= 100.0                      # 10000 huge entries in three tiles
    r0 = (0.1 * rng.standard_normal(d)).astype(np.float32)
    note("fallback after early zeros")
    routes = _check_table(gpu, oracle, [(0, d, rho)], g, r0, 1.0)
    assert routes == [2], routes
    # and the same layer without the cluster stays on the single-pass route
    g2 = rng.standard_normal(d).astype(np.float32)
    assert _check_table(gpu, oracle, [(0, d, rho)], g2, r0, 1.0) == [1]


def test_mixed_routes_in_one_table(gpu, oracle):
    """One table whose layers take all four routes at once, over several iterations."""
    rng = np.random.default_rng(53)
    sizes = [(100, 0.01), (200_000, 0.002), (60_000, 0.6), (150_000, 0.001), (6000, 0.001), (1_200_000, 0.003)]
    layers, off = [], 0
    for d, rho in sizes:
        layers.append((off, d, rho))
        off += d + 3
    table = gpu.ctx.table(layers)
    res_g = np.zeros(off, np.float32)
    res_c = np.zeros(off, np.float32)
    for it in range(4):
        g = rng.standard_normal(off).astype(np.float32)
        g[layers[3][0]:layers[3][0] + layers[3][1]] = 0.0 if it < 2 else 1.0     # zero layer -> fallback
        note("mixed routes iteration %d" % it)
        wi, wv = oracle_model_parallel(oracle, layers, g, res_c, 0.1)
        gi, gv, res_g = gpu.sparsify_model(layers, g, res_g, 0.1, table=table)
        routes = gpu.ctx.lags_last_routes(table)
        assert_same("idx", gi, wi)
        assert_same("val", gv, wv)
        assert_same("res", res_g, res_c)
        assert routes[0] == 0 and routes[4] == 0 and routes[1] == 1 and routes[5] == 1 and routes[2] == 3
        assert routes[3] == 2
    table.destroy()


def test_random_tables(gpu, oracle):
    """Seeded random tables: layer sizes across all routes, densities from 1e-4 to 1, arbitrary
    offsets with gaps, several value distributions, three iterations with error feedback,
    sparsify + merge + apply against the oracle."""
    kinds = ["normal", "ties", "mostly_zero", "narrow", "denormal", "zeros"]
    for case in range(12):
        rng = np.random.default_rng(1000 + case)
        n = int(rng.integers(1, 9))
        layers, off = [], int(rng.integers(0, 5))
        for _ in range(n):
            d = int(rng.choice([rng.integers(1, 50), rng.integers(50, 9000), rng.integers(9000, 45000),
                                rng.integers(45000, 400000)]))
            rho = float(rng.choice([1e-4, 1e-3, 5e-3, 0.03, 0.15, 0.6, 1.0]))
            layers.append((off, d, rho))
            off += d + int(rng.integers(0, 4))
        total = off + 2
        P = int(rng.integers(1, 5))
        table = gpu.ctx.table(layers)
        K = table.total_k
        res_g = [np.zeros(total, np.float32) for _ in range(P)]
        res_c = [np.zeros(total, np.float32) for _ in range(P)]
        for it in range(3):
            all_i, all_v = np.empty(P * K, np.int32), np.empty(P * K, np.float32)
            for p in range(P):
                g = np.zeros(total, np.float32)
                for (o, d, _) in layers:
                    g[o:o + d] = _values(str(rng.choice(kinds)), d, rng)
                note("random table %d iteration %d worker %d: %r" % (case, it, p, layers))
                wi, wv = oracle_model_parallel(oracle, layers, g, res_c[p], 0.25)
                gi, gv, res_g[p] = gpu.sparsify_model(layers, g, res_g[p], 0.25, table=table)
                assert_same("idx case=%d it=%d p=%d" % (case, it, p), gi, wi)
                assert_same("val case=%d it=%d p=%d" % (case, it, p), gv, wv)
                assert_same("res case=%d it=%d p=%d" % (case, it, p), res_g[p], res_c[p])
                all_i[p * K:(p + 1) * K], all_v[p * K:(p + 1) * K] = gi, gv
            want_u = np.full(total, 9.0, np.float32)
            oracle.merge_sparse(layers, all_i, all_v, P, K, want_u)
            assert_same("update case=%d" % case, gpu.merge(layers, all_i, all_v, P, K, total, table=table, fill=9.0),
                        want_u)
            param = rng.standard_normal(total).astype(np.float32)
            want_v = param.copy()
            oracle.apply_sparse(layers, all_i, all_v, P, K, want_v)
            assert_same("param case=%d" % case, gpu.apply(layers, all_i, all_v, P, K, param, table=table), want_v)
        table.destroy()


def _large_values(kind, d, rng):
    if kind == "laplace":
        return rng.laplace(size=d).astype(np.float32)
    if kind == "sparse":                      # 3 % non-zero
        x = rng.standard_normal(d).astype(np.float32)
        x[rng.random(d) < 0.97] = 0.0
        return x
    if kind == "clustered":                   # 50000 consecutive entries 80 times larger
        x = rng.standard_normal(d).astype(np.float32)
        s = int(rng.integers(0, max(1, d - 50000)))
        x[s:s + 50000] *= 80.0
        return x
    if kind == "rows":                        # four of five rows of 1500 are zero (an embedding gradient)
        x = rng.standard_normal(d).astype(np.float32)
        x[(np.arange(d) // 1500) % 5 != 0] = 0.0
        return x
    return _values(kind, d, rng)


def test_random_tables_of_large_layers(gpu, oracle):
    """Seeded random tables of layers between 41,000 and 9 million elements (the large sample for
    k >= 8192, candidate lists of every size class, rejected guesses, layers that are not sampled),
    unaligned offsets, eight value distributions, two iterations with error feedback."""
    kinds = ["normal", "laplace", "ties", "sparse", "narrow", "zeros", "clustered", "rows"]
    seen = set()
    for case in range(8):
        rng = np.random.default_rng(9100 + case)
        n = int(rng.integers(1, 4))
        layers, off = [], int(rng.integers(0, 3)) * 4
        for _ in range(n):
            d = int(rng.choice([rng.integers(41000, 300000), rng.integers(1 << 20, 3 << 20),
                                rng.integers(3 << 20, 9 << 20)]))
            rho = float(rng.choice([1e-4, 1e-3, 2e-3, 5e-3, 0.01, 0.03, 0.1, 0.3]))
            layers.append((off, d, rho))
            off += d + int(rng.integers(0, 3)) * 4
        total = off
        table = gpu.ctx.table(layers)
        res_g, res_c = np.zeros(total, np.float32), np.zeros(total, np.float32)
        for it in range(2):
            g = np.zeros(total, np.float32)
            for (o, d, _) in layers:
                g[o:o + d] = _large_values(str(rng.choice(kinds)), d, rng)
            note("large random table %d iteration %d: %r" % (case, it, layers))
            wi, wv = oracle_model_parallel(oracle, layers, g, res_c, 0.5)
            gi, gv, res_g = gpu.sparsify_model(layers, g, res_g, 0.5, table=table)
            assert_same("idx case=%d it=%d" % (case, it), gi, wi)
            assert_same("val case=%d it=%d" % (case, it), gv, wv)
            assert_same("res case=%d it=%d" % (case, it), res_g, res_c)
            seen.update(gpu.ctx.lags_last_routes(table))
        table.destroy()
    assert {1, 2, 3} <= seen, seen       # every route of the large path was taken


def test_merge_closed_forms(gpu, oracle):
    """P = 1 is a scatter; many workers on one index sum in worker order; division is a
    true division (P = 3, 7); indices spread over several merge tiles; P beyond one batch of 256."""
    rng = np.random.default_rng(31)
    layers = [(0, 20000, 0.01), (20004, 9, 0.5), (20013, 70000, 0.002)]
    total = 20013 + 70000
    K = oracle.total_k(layers)
    for P in (1, 2, 3, 7, 16, 70, 300):
        idx = np.empty(P * K, np.int32)
        val = (rng.standard_normal(P * K) * 10.0 ** rng.integers(-8, 8, P * K)).astype(np.float32)
        for p in range(P):
            pos = 0
            for (_, d, rho) in layers:
                k = oracle.topk_count(d, rho)
                hot = np.arange(k // 2)                       # shared by all workers -> P-term sums
                rest = rng.choice(np.arange(k // 2, d), k - k // 2, replace=False)
                idx[p * K + pos:p * K + pos + k] = np.sort(np.concatenate([hot, rest]))
                pos += k
        note("merge closed forms P=%d" % P)
        want = np.full(total, 123.0, np.float32)
        oracle.merge_sparse(layers, idx, val, P, K, want)
        got = gpu.merge(layers, idx, val, P, K, total)
        assert_same("update P=%d" % P, got, want)
        param = rng.standard_normal(total).astype(np.float32)
        param[::5] = -0.0
        want_v = param.copy()
        oracle.apply_sparse(layers, idx, val, P, K, want_v)
        assert_same("param P=%d" % P, gpu.apply(layers, idx, val, P, K, param), want_v)
        res = rng.standard_normal(P * total).astype(np.float32)
        assert_delta_close("delta P=%d" % P, gpu.delta(layers, res, total, idx, val, P, K),
                           oracle.delta_monitor(layers, res, total, idx, val, P, K))


def test_merge_subnormal_results(gpu, oracle):
    """Sums whose quotient by P is subnormal or rounds at the last subnormal bit, for worker
    counts that are powers of two (scaled by 1/P in the kernel) and that are not."""
    rng = np.random.default_rng(63)
    layers = [(0, 5000, 0.01)]
    K = oracle.total_k(layers)
    for P in (2, 3, 4, 16, 24, 64):
        idx = np.tile(np.sort(rng.choice(5000, K, replace=False)).astype(np.int32), P)
        val = (rng.integers(-40, 41, P * K).astype(np.float64) * 2.0 ** -149).astype(np.float32)
        val[::7] = np.float32(1.1754944e-38) * rng.standard_normal(len(val[::7])).astype(np.float32)
        val[::11] = -0.0          # 0 + (-0) is +0 whichever worker comes first
        note("merge subnormal P=%d" % P)
        want = np.empty(5000, np.float32)
        oracle.merge_sparse(layers, idx, val, P, K, want)
        assert_same("update P=%d" % P, gpu.merge(layers, idx, val, P, K, 5000), want)
        param = (rng.integers(-5, 6, 5000).astype(np.float64) * 2.0 ** -149).astype(np.float32)
        want_v = param.copy()
        oracle.apply_sparse(layers, idx, val, P, K, want_v)
        assert_same("param P=%d" % P, gpu.apply(layers, idx, val, P, K, param), want_v)


def test_apply_and_delta_edge_layers(gpu, oracle):
    """Layers of one element, k == d (delta is NaN), gaps and unaligned offsets, a padded pair
    stride and a padded worker stride; parameters outside the layers keep their bits."""
    rng = np.random.default_rng(61)
    layers = [(3, 1, 1.0), (5, 10, 1.0), (17, 9000, 0.01), (9020, 8192, 0.001), (17220, 3, 0.5)]
    total = 17230
    P, K = 5, oracle.total_k(layers)
    stride_k, res_stride = K + 3, total + 7
    idx = np.full(P * stride_k, -5, np.int32)
    val = np.full(P * stride_k, np.nan, np.float32)
    res = rng.standard_normal(P * res_stride).astype(np.float32)
    for p in range(P):
        pos = 0
        for (off, d, rho) in layers:
            k = oracle.topk_count(d, rho)
            idx[p * stride_k + pos:p * stride_k + pos + k] = np.sort(rng.choice(d, k, replace=False))
            val[p * stride_k + pos:p * stride_k + pos + k] = rng.standard_normal(k)
            pos += k
    param = rng.standard_normal(total).astype(np.float32)
    note("apply/delta edge layers")
    want_v = param.copy()
    oracle.apply_sparse(layers, idx, val, P, stride_k, want_v)
    assert_same("param", gpu.apply(layers, idx, val, P, stride_k, param), want_v)
    want_d = oracle.delta_monitor(layers, res, res_stride, idx, val, P, stride_k)
    got_d = gpu.delta(layers, res, res_stride, idx, val, P, stride_k)
    assert np.isnan(want_d[0, 2]) and np.isnan(want_d[1, 2])
    assert_delta_close("delta", got_d, want_d)


def test_determinism_and_scratch_independence(gpu, oracle):
    """Same inputs twice, with another table's work in between, give the same bits."""
    rng = np.random.default_rng(41)
    layers = [(0, 300000, 0.003), (300000, 50000, 0.01), (350000, 500, 0.1)]
    total = 350500
    g = rng.standard_normal(total).astype(np.float32)
    r0 = rng.standard_normal(total).astype(np.float32)
    a = gpu.sparsify_model(layers, g, r0, 0.1)
    gpu.sparsify_layer(rng.standard_normal(123457).astype(np.float32), np.zeros(123457, np.float32), 1.0, 999)
    b = gpu.sparsify_model(layers, g, r0, 0.1)
    for x, y, n in zip(a, b, ("idx", "val", "res")):
        assert_same(n, x, y)


def test_invalid_arguments_leave_outputs_untouched(gpu):
    import torch
    from paper_1911_08727_amd import lags
    t = torch
    g = t.zeros(100, device=gpu.dev)
    r = t.ones(100, device=gpu.dev)
    oi = t.full((5,), -7, dtype=t.int32, device=gpu.dev)
    ov = t.full((5,), 9.0, device=gpu.dev)
    for kwargs in (dict(k=0), dict(k=101), dict(lr=float("inf")), dict(lr=float("nan"))):
        with pytest.raises(lags.LagsError):
            gpu.ctx.lags_sparsify_layer(g, r, kwargs.get("lr", 0.1), kwargs.get("k", 5), oi, ov)
    with pytest.raises(lags.LagsError):                       # grad and residual overlap
        gpu.ctx.lags_sparsify_layer(g, g, 0.1, 5, oi, ov)
    with pytest.raises(lags.LagsError):                       # overlapping layers
        gpu.ctx.table([(0, 10, 0.1), (5, 10, 0.1)])
    with pytest.raises(lags.LagsError):                       # density outside (0, 1]
        gpu.ctx.table([(0, 10, 0.0)])
    t.cuda.synchronize()
    assert (oi == -7).all() and (ov == 9.0).all() and (r == 1.0).all()
