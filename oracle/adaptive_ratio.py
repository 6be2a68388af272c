"""CPU oracle of the layer-wise adaptive ratio choice (Section 5, Eq. 9 of the LAGS-SGD paper).

TEST INFRASTRUCTURE ONLY: imported by tests/ and by the benchmark's reporting of this row.
The GPU library and its binding never import it.  Plain Python floats (IEEE-754 binary64),
pure-Python loops: meant for small layers.

Eq. 9 picks, per layer l, the smallest compression ratio c = d/k whose sparse exchange
(time t_comm(c)) plus the sparsification overhead t_spar fits into the backpropagation time of
the layer computed next, t_comp^(l-1), capped by an upper bound c_u.  The printed outer "max"
with an UPPER bound is read as "min"; an empty set gives c_u.  The communication model
(Section 5 leaves the collective's cost model open) is a ring all-gather of one
message of k (index, value) pairs of 8 bytes per worker: (P-1) * (alpha + 8*k*beta).
"""
import math


def allgather_seconds(alpha, beta, P, k):
    """Ring all-gather among P workers of k 8-byte pairs each: P-1 steps of one message."""
    return float(P - 1) * (alpha + (8.0 * float(k)) * beta)


def adaptive_k(d, budget, t_spar, c_u, alpha, beta, P):
    """The definition, by exhaustion: walk k from d down to 1, i.e. c = d/k upwards from 1, and
    stop at the first ratio whose exchange is hidden; cap the ratio at c_u."""
    k_fit = 0
    for k in range(d, 0, -1):
        if allgather_seconds(alpha, beta, P, k) + t_spar <= budget:
            k_fit = k
            break
    k_cap = min(d, max(1, int(math.ceil(float(d) / c_u))))    # d/k <= c_u
    return max(k_fit, k_cap)


def adaptive_ratios(d, t_comp, t_spar, c_u, alpha, beta, P):
    """Per layer (forward order): layer l hides behind the backpropagation of layer l-1;
    layer 0, computed last, has no time to hide behind."""
    out = []
    for l in range(len(d)):
        budget = 0.0 if l == 0 else t_comp[l - 1]
        out.append(adaptive_k(d[l], budget, t_spar[l], c_u, alpha, beta, P))
    return out
