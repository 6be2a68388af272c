"""The layer-wise adaptive ratio choice (Section 5, Eq. 9; host logic, no GPU).

First the oracle (oracle/adaptive_ratio.py, exhaustive search) is pinned to what the equation and
the arithmetic fix: a hand-worked example, the closed-form inversion of the linear
communication model on exactly representable numbers, limiting cases, monotonicity.  Then the
library's lags_adaptive_ratios (bisection in C++) must agree with the oracle exactly.
"""
import math
import os

import numpy as np
import pytest

from oracle import adaptive_ratio as ora


# ---------------------------------------------------------------- pins of the oracle
def test_hand_worked_example():
    # alpha = 1, 8*beta = 1, P = 3: t_comm(k) = 2 * (1 + k).  Budget 21, t_spar 1:
    # 2 (1 + k) + 1 <= 21  <=>  k <= 9, so c = 100/9 = 11.1 (below c_u = 1000).
    assert ora.allgather_seconds(1.0, 0.125, 3, 9) == 20.0
    assert ora.adaptive_k(100, 21.0, 1.0, 1000.0, 1.0, 0.125, 3) == 9
    # a cap c_u = 5 forces k >= 20
    assert ora.adaptive_k(100, 21.0, 1.0, 5.0, 1.0, 0.125, 3) == 20
    # nothing fits (budget below the start-up cost): ratio c_u, k = ceil(d / c_u)
    assert ora.adaptive_k(100, 1.5, 0.0, 40.0, 1.0, 0.125, 3) == 3
    # everything fits: c = 1
    assert ora.adaptive_k(100, 1e9, 1.0, 1000.0, 1.0, 0.125, 3) == 100


def test_closed_form_inversion_on_exact_numbers():
    """With powers of two every product and sum below is exact, so the largest k that fits is
    floor(((budget - t_spar) / (P - 1) - alpha) / (8 beta)) exactly."""
    rng = np.random.default_rng(7)
    for _ in range(300):
        P = int(rng.choice([2, 3, 5, 9, 17]))
        alpha = float(2.0 ** rng.integers(-4, 3))
        beta = float(2.0 ** rng.integers(-8, -2))
        t_spar = float(rng.integers(0, 8)) * 0.25
        budget = float(rng.integers(0, 4000)) * 0.25
        d = int(rng.integers(1, 400))
        c_u = float(rng.choice([1.0, 2.0, 7.5, 1000.0]))
        want_fit = math.floor(((budget - t_spar) / (P - 1) - alpha) / (8 * beta))
        want_fit = max(0, min(d, want_fit))
        k_cap = min(d, max(1, math.ceil(d / c_u)))
        assert ora.adaptive_k(d, budget, t_spar, c_u, alpha, beta, P) == max(want_fit, k_cap)


def test_limits_and_monotonicity():
    # one worker communicates nothing: the exchange always fits unless t_spar alone is too long
    assert ora.adaptive_k(50, 1.0, 0.5, 1000.0, 3.0, 1.0, 1) == 50
    assert ora.adaptive_k(50, 1.0, 1.5, 1000.0, 3.0, 1.0, 1) == 1
    # a larger budget never lowers k; a slower network, a longer t_spar or more workers never raise it
    base = dict(d=300, budget=5e-3, t_spar=1e-4, c_u=1000.0, alpha=5e-5, beta=1e-6, P=8)
    k0 = ora.adaptive_k(**base)
    assert 1 < k0 < 300
    for key, factor, sign in (("budget", 1.3, +1), ("alpha", 1.3, -1), ("beta", 1.3, -1), ("t_spar", 5.0, -1)):
        kw = dict(base)
        kw[key] = base[key] * factor
        assert (ora.adaptive_k(**kw) - k0) * sign >= 0, key
    assert ora.adaptive_k(**dict(base, P=16)) <= k0
    # the chosen k satisfies the inequality and k + 1 does not
    t = lambda k: ora.allgather_seconds(base["alpha"], base["beta"], base["P"], k) + base["t_spar"]
    assert t(k0) <= base["budget"] < t(k0 + 1)


def test_layer_pipeline_order():
    """Layer l hides behind layer l-1; layer 0 has no budget and gets the capped ratio."""
    d = [64, 1000, 1000]
    t_comp = [4.0, 0.0, 123.0]
    ks = ora.adaptive_ratios(d, t_comp, [0.0, 0.0, 0.0], 500.0, 0.0, 0.125, 2)
    assert ks[0] == 1                       # no budget: ceil(64 / 500)
    assert ks[1] == 4                       # budget 4.0 = t_comp[0]: 1 * k <= 4 (above the cap's 2)
    assert ks[2] == 2                       # budget 0.0 = t_comp[1]: nothing fits (k >= 1 costs 1) -> ceil(1000 / 500)


# ---------------------------------------------------------------- the library against the oracle
@pytest.fixture(scope="module")
def lags():
    from paper_1911_08727_amd import build, lags
    if not os.path.exists(lags.LIB_PATH):
        build.build()
    return lags


def test_library_matches_oracle_on_random_tables(lags, oracle):
    rng = np.random.default_rng(11)
    for case in range(120):
        n = int(rng.integers(1, 9))
        d = [int(rng.choice([rng.integers(1, 20), rng.integers(20, 3000), rng.integers(3000, 40000)])) for _ in range(n)]
        P = int(rng.choice([1, 2, 4, 16, 64]))
        alpha = float(rng.choice([0.0, 1e-6, 5e-5, 1e-3]))
        beta = float(rng.choice([0.0, 1e-10, 8e-10, 1e-7]))
        c_u = float(rng.choice([1.0, 4.0, 250.0, 1000.0, 1e6]))
        t_comp = [float(x) for x in rng.choice([0.0, 1e-5, 3e-4, 2e-3, 0.05], n)]
        t_spar = [float(x) for x in rng.choice([0.0, 1e-6, 1e-4, 1e-2], n)]
        got_k, got_rho = lags.lags_adaptive_ratios(alpha, beta, P, d, t_comp, t_spar, c_u)
        want = ora.adaptive_ratios(d, t_comp, t_spar, c_u, alpha, beta, P)
        assert got_k == want, (case, d, P, alpha, beta, c_u, t_comp, t_spar)
        for dl, kl, rl in zip(d, got_k, got_rho):
            assert 0.0 < rl <= 1.0
            assert lags.lags_topk_count(dl, rl) == kl          # the density reproduces k in the library
            assert oracle.topk_count(dl, rl) == kl             # ... and in the oracle's own rule


def test_library_communication_model_is_the_oracles(lags):
    rng = np.random.default_rng(12)
    for _ in range(200):
        a, b = float(rng.random() * 1e-3), float(rng.random() * 1e-8)
        P, k = int(rng.integers(1, 1025)), int(rng.integers(0, 1 << 31))
        assert lags.lags_allgather_seconds(a, b, P, k) == ora.allgather_seconds(a, b, P, k)
    assert math.isnan(lags.lags_allgather_seconds(1.0, 1.0, 0, 5))


def test_density_round_trip_at_large_sizes(lags, oracle):
    """rho_out must give back k for every (d, k), also where k/d rounds upwards."""
    rng = np.random.default_rng(13)
    for _ in range(400):
        d = int(rng.choice([rng.integers(1, 1000), rng.integers(1000, 1 << 20), rng.integers(1 << 20, (1 << 31) - 1)]))
        # force a chosen k through the cap: nothing fits, k = ceil(d / c_u)
        k_target = int(rng.integers(1, d + 1))
        c_u = d / k_target
        if c_u < 1.0:
            continue
        ks, rhos = lags.lags_adaptive_ratios(1.0, 1.0, 2, [d], [0.0], [0.0], c_u)
        assert ks[0] == min(d, max(1, math.ceil(d / c_u)))
        assert lags.lags_topk_count(d, rhos[0]) == ks[0]
        assert oracle.topk_count(d, rhos[0]) == ks[0]


def test_library_rejects_bad_arguments(lags):
    from paper_1911_08727_amd.lags import LagsError
    good = dict(alpha=1e-5, beta=1e-9, P=4, d=[100], t_comp=[1e-3], t_spar=[1e-5], c_u=1000.0)
    lags.lags_adaptive_ratios(**good)
    for key, bad in (("P", 0), ("alpha", -1.0), ("beta", float("nan")), ("c_u", 0.5), ("d", [0]),
                     ("d", [1 << 31]), ("t_comp", [-1.0]), ("t_spar", [float("nan")])):
        with pytest.raises(LagsError):
            lags.lags_adaptive_ratios(**dict(good, **{key: bad}))


# ---------------------------------------------------------------- the pins have teeth
ORACLE_PINS = [test_hand_worked_example, test_closed_form_inversion_on_exact_numbers,
               test_limits_and_monotonicity, test_layer_pipeline_order]

ORACLE_MUTANTS = {
    "all_P_workers_send": ("return float(P - 1) *", "return float(P) *"),
    "four_bytes_per_pair": ("(8.0 * float(k))", "(4.0 * float(k))"),
    "no_startup_cost": ("(alpha + (8.0 * float(k)) * beta)", "((8.0 * float(k)) * beta)"),
    "overhead_ignored": ("+ t_spar <= budget", "<= budget"),
    "strict_inequality": ("+ t_spar <= budget", "+ t_spar < budget"),
    "smallest_k_that_fits": ("for k in range(d, 0, -1):", "for k in range(1, d + 1):"),
    "cap_is_a_lower_bound_of_the_ratio": ("return max(k_fit, k_cap)", "return min(k_fit, k_cap) if k_fit else k_cap"),
    "cap_rounded_down": ("int(math.ceil(float(d) / c_u))", "int(math.floor(float(d) / c_u))"),
    "hides_behind_its_own_backprop": ("budget = 0.0 if l == 0 else t_comp[l - 1]", "budget = t_comp[l]"),
    "hides_behind_the_layer_above": ("budget = 0.0 if l == 0 else t_comp[l - 1]",
                                     "budget = 0.0 if l == len(d) - 1 else t_comp[l + 1]"),
}


@pytest.mark.parametrize("name", sorted(ORACLE_MUTANTS))
def test_oracle_mutant_is_caught(name, monkeypatch):
    """Each plausible mistake, planted in a copy of the oracle's source, fails some pin above."""
    import sys
    import types
    old, new = ORACLE_MUTANTS[name]
    src = open(ora.__file__).read()
    assert src.count(old) == 1, "mutation site not found: %s" % name
    mutant = types.ModuleType("adaptive_ratio_mutant")
    exec(compile(src.replace(old, new), "mutant_" + name, "exec"), mutant.__dict__)
    monkeypatch.setattr(sys.modules[__name__], "ora", mutant)
    caught = False
    for pin in ORACLE_PINS:
        try:
            pin()
        except (AssertionError, ZeroDivisionError):
            caught = True
            break
    assert caught, "no pin notices mutant %s" % name
