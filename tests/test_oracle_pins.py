"""Pins of the CPU oracle against things other than itself (CPU only).

Each test states which plausible mistake in oracle/lags_oracle.c it would catch.
Paper passages: Algorithm 1 lines 6-9, Eq. 4 (TopK), Eq. 5, Section 4.2
(RandK identity used in Lemma 1).
"""
import itertools
import os
import struct
from fractions import Fraction

import numpy as np
import pytest

from exact32 import round_f32, fraction_to_bits

HERE = os.path.dirname(os.path.abspath(__file__))


def bits(a):
    return np.ascontiguousarray(a, np.float32).view(np.uint32)


def keys(a):
    return bits(a) & np.uint32(0x7FFFFFFF)


# ---------------------------------------------------------------- k ---------
def test_topk_count_golden(oracle):
    """Catches: floor instead of ceil, missing max(1, .), missing clamp to d."""
    rows = []
    for line in open(os.path.join(HERE, "golden", "topk_count.txt")):
        line = line.split("#")[0].split()
        if line:
            rows.append((int(line[0]), float(line[1]), int(line[2])))
    assert len(rows) >= 20
    for d, rho, k in rows:
        assert oracle.topk_count(d, rho) == k, (d, rho)


def test_topk_count_compression_ratio_identity(oracle):
    """c = d/k (Lemma 1): for d a multiple of c, k = d/c exactly, for the paper's c = 1000 and 250."""
    for c in (1000, 250, 200):
        for m in (1, 2, 3, 17, 1000, 4097, 102760):
            assert oracle.topk_count(c * m, 1.0 / c) in (m, m + 1)  # 1/c is not exact in binary
    for m in (1, 2, 3, 17, 1000, 4097, 102760):
        assert oracle.topk_count(1000 * m, 0.001) == m
        assert oracle.topk_count(200 * m, 0.005) == m


# --------------------------------------------------------- accumulate -------
def _exact_acc(lr, g, r):
    """fl32(r + fl32(lr*g)) computed with rationals; +-0 results returned as Fraction(0)."""
    t = round_f32(Fraction(float(lr)) * Fraction(float(g)))
    return round_f32(Fraction(float(r)) + t)


def _exact_fma(lr, g, r):
    return round_f32(Fraction(float(lr)) * Fraction(float(g)) + Fraction(float(r)))


def test_accumulate_two_roundings_exact(oracle):
    """Algorithm 1 line 6 in binary32 with two roundings.
    Catches: fused multiply-add, double-precision intermediate, swapped operands (lr*r + g)."""
    rng = np.random.default_rng(5)
    n = 4000
    g = rng.standard_normal(n).astype(np.float32)
    r = (rng.standard_normal(n) * 0.1).astype(np.float32)
    lr = np.float32(0.1)
    acc = oracle.accumulate(g, r, lr)
    n_fma_differs = 0
    for i in range(n):
        want = _exact_acc(lr, g[i], r[i])
        assert Fraction(float(acc[i])) == want, i
        if _exact_fma(lr, g[i], r[i]) != want:
            n_fma_differs += 1
    # the no-FMA requirement is only tested if some element distinguishes the two
    assert n_fma_differs > 50


def test_accumulate_handpicked_fma_case(oracle):
    """A single worked element where fma(lr, g, r) != fl(fl(lr*g) + r).
    lr = 0.1f = 13421773 * 2^-27; g = 3; r = -0.3f (= -10066330 * 2^-25).
    lr*g = 40265319 * 2^-27 exactly, which needs 26 bits: it rounds to 10066330 * 2^-25,
    so the two-rounding sum is exactly 0 while the fused result is -2^-27."""
    lr = np.float32(0.1)
    g = np.array([3.0], np.float32)
    r = np.array([-0.3], np.float32)
    assert Fraction(float(lr)) == Fraction(13421773, 2 ** 27)
    assert Fraction(float(r[0])) == -Fraction(10066330, 2 ** 25)
    acc = oracle.accumulate(g, r, lr)
    assert acc[0] == 0.0 and bits(acc)[0] == 0          # +0.0, not -0.0 and not -2^-27
    assert _exact_fma(lr, g[0], r[0]) == -Fraction(1, 2 ** 27)


def test_accumulate_keeps_denormals(oracle):
    """Catches flush-to-zero: a product in the subnormal range must survive."""
    lr = np.float32(0.5)
    g = np.array([2.0 ** -140, -(2.0 ** -149) * 6], np.float32)
    r = np.zeros(2, np.float32)
    acc = oracle.accumulate(g, r, lr)
    assert Fraction(float(acc[0])) == Fraction(1, 2 ** 141)
    assert Fraction(float(acc[1])) == -Fraction(3, 2 ** 149)


# ---------------------------------------------------- selection: brute ------
def _brute_force_set(acc, k):
    """Eq. 4 made total: the unique k-subset S such that every member precedes every
    non-member in the order (|x| descending, index ascending).  Found by enumeration."""
    d = len(acc)
    key = keys(acc)
    found = None
    for S in itertools.combinations(range(d), k):
        inS = set(S)
        ok = True
        for i in S:
            for j in range(d):
                if j in inS:
                    continue
                if not (key[i] > key[j] or (key[i] == key[j] and i < j)):
                    ok = False
                    break
            if not ok:
                break
        if ok:
            assert found is None, "order is not total"
            found = S
    assert found is not None
    return found


SPECIAL = [0.0, -0.0, 1.0, -1.0, 2.0, -2.0, 0.5, 1e-45, -1e-45, 3e-39, float("inf"), -float("inf"),
           1.0000001, -3.5]


def _value_sets():
    rng = np.random.default_rng(11)
    sets = [
        np.zeros(7, np.float32),
        np.full(6, 1.5, np.float32),
        np.array([1, -1, 1, -1, 1, -1, 1, -1], np.float32),
        np.array([0.0, -0.0, 0.0, -0.0, 1e-45], np.float32),
        np.array([3, 1, 2], np.float32),
        np.array([-5], np.float32),
        np.array([1, 2, 3, 4, 5, 6, 7, 8, 9], np.float32),
        np.array([9, 8, 7, 6, 5, 4, 3, 2, 1], np.float32),
    ]
    for d in (2, 3, 5, 8, 10):
        for _ in range(6):
            sets.append(rng.choice(np.array(SPECIAL, np.float32), d))
            sets.append(rng.integers(-2, 3, d).astype(np.float32))
            sets.append(rng.standard_normal(d).astype(np.float32))
    return sets


def test_selection_bruteforce_all_k(oracle):
    """Catches: ascending instead of descending sort, signed instead of absolute value,
    wrong tie direction, off-by-one in the number kept, output not in index order,
    value taken from grad instead of acc, residual not zeroed / zeroed at the wrong slots."""
    for acc0 in _value_sets():
        d = len(acc0)
        for k in range(1, d + 1):
            # lr = 1 and residual = -0.0 make acc == grad bit for bit (x + -0 = x, also for
            # x = -0), so the set is known up front
            res = np.full(d, -0.0, np.float32)
            idx, val = oracle.sparsify_layer(acc0.copy(), res, 1.0, k)
            S = _brute_force_set(acc0, k)
            assert tuple(idx.tolist()) == S, (acc0, k)
            assert bits(val).tolist() == bits(acc0[list(S)]).tolist()
            for i in range(d):
                if i in S:
                    assert bits(res)[i] == 0
                else:
                    assert bits(res)[i] == bits(acc0)[i]
            # the kept magnitudes are a maximal k-subset (finite cases)
            mags = np.abs(acc0.astype(np.float64))
            if np.all(np.isfinite(mags)):
                best = max(sum(mags[list(c)]) for c in itertools.combinations(range(d), k))
                assert sum(mags[list(S)]) == best


def test_selection_uses_acc_not_grad(oracle):
    """Residual changes the winner: grad alone would pick index 0, acc picks index 2."""
    g = np.array([1.0, 0.5, 0.25], np.float32)
    r = np.array([-0.9, 0.0, 0.5], np.float32)
    idx, val = oracle.sparsify_layer(g, r, 1.0, 1)
    assert idx.tolist() == [2] and val.tolist() == [0.75]
    assert r.tolist() == [np.float32(1.0) + np.float32(-0.9), 0.5, 0.0]


def test_selection_nan_ranks_first(oracle):
    g = np.array([1.0, float("nan"), float("inf"), -2.0], np.float32)
    r = np.zeros(4, np.float32)
    idx, _ = oracle.sparsify_layer(g, r, 1.0, 2)
    assert idx.tolist() == [1, 2]


# ------------------------------------------- selection: library routine -----
@pytest.mark.parametrize("d,k", [(1000, 1), (1000, 999), (4097, 41), (100003, 101), (100003, 5000)])
def test_selection_matches_partition_on_tie_free_data(oracle, d, k):
    """On data without equal magnitudes the kept set is what numpy's partition keeps."""
    rng = np.random.default_rng(d + k)
    g = rng.standard_normal(d).astype(np.float32)
    r = (0.3 * rng.standard_normal(d)).astype(np.float32)
    lr = np.float32(0.1)
    for _ in range(100):                                  # redraw only the colliding entries
        acc = (r + lr * g).astype(np.float32)             # numpy float32 ops: two roundings
        _, inv, cnt = np.unique(np.abs(acc), return_inverse=True, return_counts=True)
        dup = np.flatnonzero(cnt[inv] > 1)
        if len(dup) == 0:
            break
        g[dup] = rng.standard_normal(len(dup)).astype(np.float32)
    assert len(np.unique(np.abs(acc))) == d
    res = r.copy()
    idx, val = oracle.sparsify_layer(g, res, lr, k)
    want = np.sort(np.argpartition(-np.abs(acc), k - 1)[:k])
    assert np.array_equal(idx, want.astype(np.int32))
    assert np.array_equal(bits(val), bits(acc[want]))


# ------------------------------------------------------- invariants ---------
@pytest.mark.parametrize("seed", range(6))
def test_invariants_with_heavy_ties(oracle, seed):
    """Algorithm 1 line 7: residual + TopK == acc; exactly k kept; threshold and tie rule."""
    rng = np.random.default_rng(100 + seed)
    d = int(rng.integers(50, 3000))
    k = int(rng.integers(1, d + 1))
    g = rng.integers(-3, 4, d).astype(np.float32)       # few distinct magnitudes -> many ties
    r = (rng.integers(-2, 3, d) * 0.5).astype(np.float32)
    lr = np.float32(0.5)
    acc = (r + lr * g).astype(np.float32)
    res = r.copy()
    idx, val = oracle.sparsify_layer(g, res, lr, k)
    assert len(idx) == k and np.all(np.diff(idx) > 0)
    sel = np.zeros(d, bool)
    sel[idx] = True
    ky = keys(acc)
    T = ky[sel].min()
    assert ky[~sel].max(initial=0) <= T
    # among entries equal to the threshold the lowest indices are the ones kept
    ties = np.flatnonzero(ky == T)
    n_taken = int(sel[ties].sum())
    assert np.array_equal(np.flatnonzero(sel[ties]), np.arange(n_taken))
    assert np.all(sel[ky > T])
    dense = np.zeros(d, np.float32)
    dense[idx] = val
    assert np.array_equal(bits(np.where(sel, dense, res)), bits(acc))
    assert np.all(bits(res)[sel] == 0)


def test_energy_bound_of_randk(oracle):
    """Section 4.2: E||x - RandK(x,k)||^2 = (1 - k/d)||x||^2, and TopK is at least as good."""
    rng = np.random.default_rng(9)
    for d, k in ((1000, 1), (1000, 10), (5000, 2500), (333, 332)):
        g = rng.standard_normal(d).astype(np.float32)
        res = np.zeros(d, np.float32)
        oracle.sparsify_layer(g, res, 1.0, k)
        lhs = float(np.sum(res.astype(np.float64) ** 2))
        rhs = (1.0 - k / d) * float(np.sum(g.astype(np.float64) ** 2))
        assert lhs <= rhs * (1 + 1e-12)


# ------------------------------------------------------------ model ---------
def test_model_is_layerwise_and_packs_outputs(oracle):
    """Layer-wise selection (Section 4.1): each layer keeps its own k_l entries with
    layer-local indices, packed one layer after the other."""
    rng = np.random.default_rng(21)
    layers = [(0, 10, 0.2), (10, 7, 0.5), (20, 33, 0.1)]          # a gap between layer 1 and 2
    g = rng.standard_normal(53).astype(np.float32)
    r0 = rng.standard_normal(53).astype(np.float32)
    r = r0.copy()
    idx, val = oracle.sparsify_model(layers, g, r, 0.25)
    pos = 0
    for off, d, rho in layers:
        k = oracle.topk_count(d, rho)
        rl = r0[off:off + d].copy()
        li, lv = oracle.sparsify_layer(g[off:off + d].copy(), rl, 0.25, k)
        assert np.array_equal(idx[pos:pos + k], li) and np.array_equal(bits(val[pos:pos + k]), bits(lv))
        assert np.array_equal(bits(r[off:off + d]), bits(rl))
        pos += k
    assert pos == len(idx)
    assert np.array_equal(bits(r[17:20]), bits(r0[17:20]))          # the gap is untouched
    # a model-wide top-k would differ: the largest |acc| of layer 2 are not all kept
    assert pos == 2 + 4 + 4


# ------------------------------------------------------------ merge ---------
def test_merge_single_worker_is_scatter(oracle):
    layers = [(0, 8, 0.25), (8, 5, 0.4)]
    idx = np.array([1, 6, 0, 4], np.int32)
    val = np.array([2.0, -3.0, 0.5, 7.0], np.float32)
    upd = np.full(13, 99.0, np.float32)
    oracle.merge_sparse(layers, idx, val, 1, 4, upd)
    want = np.zeros(13, np.float32)
    want[[1, 6, 8, 12]] = [2.0, -3.0, 0.5, 7.0]
    assert np.array_equal(bits(upd), bits(want))


def test_merge_disjoint_and_identical_supports(oracle):
    """Algorithm 1 lines 8-9: g = sum_p TopK_p, update = g / P."""
    layers = [(0, 10, 0.2)]
    P = 4
    idx = np.array([0, 1, 2, 3, 4, 5, 6, 7], np.int32)
    val = np.array([1, 2, 3, 4, 5, 6, 7, 8], np.float32)
    upd = np.empty(10, np.float32)
    oracle.merge_sparse(layers, idx, val, P, 2, upd)
    want = np.zeros(10, np.float32)
    want[:8] = val / np.float32(4)
    assert np.array_equal(bits(upd), bits(want))
    idx = np.tile(np.array([3, 9], np.int32), P)
    val = np.tile(np.array([0.1, -0.7], np.float32), P)
    oracle.merge_sparse(layers, idx, val, P, 2, upd)
    want = np.zeros(10, np.float32)
    for j, v in ((3, 0.1), (9, -0.7)):
        s = Fraction(0)
        for _ in range(P):
            s = round_f32(s + Fraction(float(np.float32(v))))
        want[j] = float(round_f32(s / P))
    assert np.array_equal(bits(upd), bits(want))


def test_merge_order_and_true_division(oracle):
    """Sum runs p = 0,1,2 in that order, then one division by P (not a multiply by fl(1/P)).
    Catches: reversed/pairwise order, per-term division, reciprocal multiply, stride misuse."""
    layers = [(0, 4, 0.5)]
    P = 3
    # stride_k = 3 > k = 2: one padding slot between the workers' blocks
    idx = np.array([0, 2, -1, 0, 2, -1, 0, 2, -1], np.int32)
    val = np.array([1e8, 4.0, 777, -1e8, 2.0, 777, 1.0, 1.0, 777], np.float32)
    upd = np.empty(4, np.float32)
    oracle.merge_sparse(layers, idx, val, P, 3, upd)
    assert Fraction(float(upd[0])) == round_f32(Fraction(1, 3))        # (1e8 - 1e8) + 1, / 3
    assert Fraction(float(upd[2])) == round_f32(Fraction(7, 3))        # (4 + 2 + 1) / 3
    # 7 * fl(1/3) rounds differently: the division must be a true division
    assert round_f32(Fraction(7) * round_f32(Fraction(1, 3))) != round_f32(Fraction(7, 3))
    assert bits(upd)[1] == 0 and bits(upd)[3] == 0


def test_merge_leaves_gaps_alone(oracle):
    layers = [(2, 3, 0.3), (8, 2, 0.5)]
    idx = np.array([1, 0], np.int32)
    val = np.array([4.0, -6.0], np.float32)
    upd = np.full(12, 5.0, np.float32)
    oracle.merge_sparse(layers, idx, val, 1, 2, upd)
    assert upd.tolist() == [5, 5, 0, 4, 0, 5, 5, 5, -6, 0, 5, 5]


# ---------------------------------------------------- multi-iteration -------
def test_error_feedback_conserves_mass(oracle):
    """Algorithm 1 lines 6-7 over T iterations: sum_t TopK_t + residual_T = sum_t lr*grad_t
    (up to binary32 rounding; checked in float64)."""
    rng = np.random.default_rng(77)
    d, k, lr, T = 5000, 50, np.float32(0.1), 12
    res = np.zeros(d, np.float32)
    sent = np.zeros(d, np.float64)
    total = np.zeros(d, np.float64)
    for _ in range(T):
        g = rng.standard_normal(d).astype(np.float32)
        total += float(lr) * g.astype(np.float64)
        idx, val = oracle.sparsify_layer(g, res, lr, k)
        sent[idx] += val
    assert np.allclose(sent + res, total, rtol=0, atol=1e-5)
    # and the feedback matters: without the residual the kept set of the last step differs
    res2 = np.zeros(d, np.float32)
    idx2, _ = oracle.sparsify_layer(g, res2, lr, k)
    assert not np.array_equal(idx, idx2)


# ------------------------------------------------------ sparse apply --------
def test_apply_single_worker_and_untouched_entries(oracle):
    """Algorithm 1 line 9 with P = 1: v - TopK; entries no worker selected keep their bits
    (also -0.0 and denormals)."""
    layers = [(1, 6, 0.5), (8, 3, 0.3)]
    idx = np.array([0, 2, 5, 1], np.int32)
    val = np.array([0.5, -2.0, 4.0, 8.0], np.float32)
    v0 = np.array([9, 1.0, -0.0, 3.0, 1e-45, 0.0, 7.0, 9, 2.0, 2.0, -0.0, 9], np.float32)
    v = v0.copy()
    oracle.apply_sparse(layers, idx, val, 1, 4, v)
    want = v0.copy()
    want[1] = 1.0 - 0.5
    want[3] = 3.0 + 2.0
    want[6] = 7.0 - 4.0
    want[9] = 2.0 - 8.0
    assert np.array_equal(bits(v), bits(want))


def test_apply_sums_then_divides_then_subtracts(oracle):
    """v_new = fl(v - fl(fl(a + b + c) / P)): one rounding per step, in that order.
    Catches: subtracting per worker, multiplying by fl(1/P), adding instead of subtracting."""
    layers = [(0, 2, 0.5)]
    P = 3
    found = 0
    rng = np.random.default_rng(17)
    for _ in range(200):
        a, b, c, v0 = [np.float32(x) for x in rng.standard_normal(4)]
        idx = np.zeros(P, np.int32)
        val = np.array([a, b, c], np.float32)
        v = np.array([v0, 5.0], np.float32)
        oracle.apply_sparse(layers, idx, val, P, 1, v)
        s = round_f32(round_f32(Fraction(float(a)) + Fraction(float(b))) + Fraction(float(c)))
        want = round_f32(Fraction(float(v0)) - round_f32(s / 3))
        assert Fraction(float(v[0])) == want and v[1] == 5.0
        per_worker = Fraction(float(v0))
        for x in (a, b, c):
            per_worker = round_f32(per_worker - round_f32(Fraction(float(x)) / 3))
        recip = round_f32(Fraction(float(v0)) - round_f32(s * round_f32(Fraction(1, 3))))
        found += (per_worker != want) + (recip != want)
    assert found > 20        # the alternatives really do round differently on these inputs


# ------------------------------------------------------ delta monitor -------
def test_delta_hand_example(oracle):
    """Section 6.2 on a 4-element layer, two workers, k = 2, worked by hand:
    residual sums (1,0,1,3) -> numerator 11; x sums (6,-1,3,3) -> 55; delta = 11 / (0.5*55)."""
    res = np.array([0, 0, 1, 2, 1, 0, 0, 1], np.float32)
    idx = np.array([0, 1, 1, 2], np.int32)
    val = np.array([5, -4, 3, 2], np.float32)
    out = oracle.delta_monitor([(0, 4, 0.5)], res, 4, idx, val, 2, 2)
    assert out.tolist() == [[11.0, 55.0, 0.4]]


def test_delta_from_definition_and_randk_identity(oracle):
    """delta from (new residuals, selected pairs) equals the definition evaluated on the acc
    vectors with numpy, and its denominator is the RandK expectation of Section 4.2, checked by
    exhaustive enumeration of all k-subsets on a tiny vector."""
    rng = np.random.default_rng(23)
    P, d, k = 5, 400, 20
    layers = [(0, d, k / d)]
    accs = rng.standard_normal((P, d)).astype(np.float32)
    res = np.empty((P, d), np.float32)
    idx = np.empty((P, k), np.int32)
    val = np.empty((P, k), np.float32)
    for p in range(P):
        r = np.full(d, -0.0, np.float32)
        idx[p], val[p] = oracle.sparsify_layer(accs[p].copy(), r, 1.0, k)
        res[p] = r
    out = oracle.delta_monitor(layers, res.reshape(-1), d, idx.reshape(-1), val.reshape(-1), P, k)
    x = accs.astype(np.float64)
    top = np.zeros_like(x)
    for p in range(P):
        keep = np.argpartition(-np.abs(x[p]), k - 1)[:k]
        top[p, keep] = x[p, keep]
    num = float(np.sum((x.sum(0) - top.sum(0)) ** 2))
    sq = float(np.sum(x.sum(0) ** 2))
    assert np.isclose(out[0, 0], num, rtol=1e-12) and np.isclose(out[0, 1], sq, rtol=1e-12)
    assert np.isclose(out[0, 2], num / ((1 - k / d) * sq), rtol=1e-12)
    assert out[0, 2] < 1.0                      # what the paper observes (Fig. 2)
    # E || y - RandK(y, k) ||^2 = (1 - k/d) ||y||^2 by enumeration
    y = rng.standard_normal(7)
    for kk in (1, 3, 6):
        errs = [np.sum(np.delete(y, list(c)) ** 2) for c in itertools.combinations(range(7), kk)]
        assert np.isclose(np.mean(errs), (1 - kk / 7) * np.sum(y ** 2))


def test_delta_single_worker_bound_and_full_density(oracle):
    """P = 1: TopK is at least as good as RandK, so delta <= 1; k = d: denominator 0 -> NaN."""
    rng = np.random.default_rng(29)
    d = 1000
    g = rng.standard_normal(d).astype(np.float32)
    for k in (1, 10, 500):
        r = np.zeros(d, np.float32)
        i, v = oracle.sparsify_layer(g, r, 1.0, k)
        out = oracle.delta_monitor([(0, d, k / d)], r, d, i, v, 1, k)
        assert 0.0 <= out[0, 2] <= 1.0
    r = np.zeros(d, np.float32)
    i, v = oracle.sparsify_layer(g, r, 1.0, d)
    out = oracle.delta_monitor([(0, d, 1.0)], r, d, i, v, 1, d)
    assert out[0, 0] == 0.0 and np.isnan(out[0, 2])


def test_delta_uses_layer_offsets_and_strides(oracle):
    """Two layers with a gap, worker stride larger than the model, pair stride larger than sum k."""
    layers = [(1, 3, 0.4), (6, 2, 0.5)]
    P = 2
    res = np.array([9, 1, 0, 2, 9, 9, 0, 1, 9, 9,
                    9, 0, 0, 1, 9, 9, 3, 0, 9, 9], np.float32)
    idx = np.array([1, 2, 0, -1, 0, 1, 1, -1], np.int32)          # k = 2, 1 ; stride_k = 4
    val = np.array([4, 1, 5, 77, 2, 2, -1, 77], np.float32)
    out = oracle.delta_monitor(layers, res, 10, idx, val, P, 4)
    # layer 0: residual sums (1,0,3) -> 10; selected sums (2,6,1) -> x = (3,6,4) -> 61
    assert out[0].tolist()[:2] == [10.0, 61.0] and np.isclose(out[0, 2], 10 / ((1 - 2 / 3) * 61))
    # layer 1: residual sums (3,1) -> 10; selected sums (5,-1) -> x = (8,0) -> 64
    assert out[1].tolist()[:2] == [10.0, 64.0] and np.isclose(out[1, 2], 10 / (0.5 * 64))


def test_apply_two_workers_strided_blocks(oracle):
    """Worker blocks sit stride_k apart (here with one padding slot), layers at their offsets."""
    layers = [(0, 4, 0.5), (5, 2, 0.5)]
    idx = np.array([0, 3, 1, -1, 0, 2, 1, -1], np.int32)            # per worker: k = 2, 1, pad
    val = np.array([2, 4, 6, 77, 10, 20, 30, 77], np.float32)
    v = np.array([1, 1, 1, 1, 9, 1, 1], np.float32)
    oracle.apply_sparse(layers, idx, val, 2, 4, v)
    assert v.tolist() == [1 - 6, 1, 1 - 10, 1 - 2, 9, 1, 1 - 18]
