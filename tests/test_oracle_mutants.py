"""The pins have teeth: each plausible mistake, planted in a copy of the oracle's source
(on the CPU, in a temporary file), is caught by at least one pin of test_oracle_pins.py."""
import os
import subprocess
import tempfile

import pytest

import oracle as oracle_pkg
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle_pkg.__file__), "lags_oracle.c")

MUTANTS = {
    "floor_instead_of_ceil": ("double x = ceil(rho * (double)d);", "double x = floor(rho * (double)d);"),
    "no_min_one": ("if (k < 1) k = 1;", ""),
    "no_clamp_to_d": ("if (k > d) k = d;", ""),
    "fused_multiply_add": ("float t = lr * grad[i];\n    acc[i] = residual[i] + t;",
                           "acc[i] = fmaf(lr, grad[i], residual[i]);"),
    "double_intermediate": ("float t = lr * grad[i];\n    acc[i] = residual[i] + t;",
                            "acc[i] = (float)((double)residual[i] + (double)lr * (double)grad[i]);"),
    "lr_on_residual": ("float t = lr * grad[i];\n    acc[i] = residual[i] + t;",
                       "float t = lr * residual[i];\n    acc[i] = grad[i] + t;"),
    "signed_key": ("return bits_of(x) & 0x7FFFFFFFu;", "return bits_of(x) ^ 0x80000000u;"),
    "ascending_magnitude": ("return a->key > b->key ? -1 : 1;", "return a->key > b->key ? 1 : -1;"),
    "ties_to_higher_index": ("return a->idx < b->idx ? -1 : 1;", "return a->idx < b->idx ? 1 : -1;"),
    "strictly_above_threshold": ("for (int64_t j = 0; j < k; ++j) selected[order[j].idx] = 1;",
                                 "for (int64_t j = 0; j + 1 < k; ++j) selected[order[j].idx] = 1;\n"
                                 "  selected[order[0].idx] = 1; if (k > 1) k -= 1;"),
    "emit_grad_value": ("out_val[n] = acc[i];", "out_val[n] = grad[i];"),
    "residual_not_zeroed": ("      residual[i] = 0.0f;\n", "      residual[i] = acc[i];\n"),
    "residual_keeps_old": ("      residual[i] = acc[i];\n    }\n  }\n  free(acc);", "    }\n  }\n  free(acc);"),
    "global_indices": ("out_idx[n] = (int32_t)i;", "out_idx[n] = (int32_t)(i + (grad - (const float*)0) % 1);"),
    "merge_reverse_order": ("for (int32_t p = 0; p < P; ++p) {", "for (int32_t p = P - 1; p >= 0; --p) {"),
    "merge_reciprocal": ("u[i] = u[i] / fp;", "u[i] = u[i] * (1.0f / fp);"),
    "merge_no_average": ("u[i] = u[i] / fp;", "u[i] = u[i];"),
    "merge_ignores_stride": ("const int32_t *pi = idx + (int64_t)p * stride_k + out;",
                             "const int32_t *pi = idx + (int64_t)p * k + out;"),
    "merge_no_clear": ("for (int64_t i = 0; i < d; ++i) u[i] = 0.0f;", ""),
    "apply_adds": ("v[i] = v[i] - update[i];", "v[i] = v[i] + update[i];"),
    "apply_ignores_stride": ("int rc = oracle_merge_sparse(&one, 1, idx + out, val + out, P, stride_k, update);",
                             "int rc = oracle_merge_sparse(&one, 1, idx + out, val + out, P, k, update);"),
    "apply_wrong_offset": ("float *v = param_flat + layers[l].offset;", "float *v = param_flat + out;"),
    "delta_no_randk_factor": ("double den = (1.0 - (double)k / (double)d) * sq;", "double den = sq;"),
    "delta_factor_k_over_d": ("double den = (1.0 - (double)k / (double)d) * sq;",
                              "double den = ((double)k / (double)d) * sq;"),
    "delta_numerator_is_x": ("num += sum_res[i] * sum_res[i];", "num += x * x;"),
    "delta_denominator_is_residual": ("sq += x * x;", "sq += sum_res[i] * sum_res[i];"),
    "delta_norm_not_squared": ("num += sum_res[i] * sum_res[i];", "num += fabs(sum_res[i]);"),
    "delta_sums_norms_per_worker": ("for (int64_t i = 0; i < d; ++i) sum_res[i] += (double)r[i];",
                                    "for (int64_t i = 0; i < d; ++i) sum_res[i] += fabs((double)r[i]);"),
    "delta_ignores_res_stride": ("const float *r = residual_flat + (int64_t)p * res_stride + layers[l].offset;",
                                 "const float *r = residual_flat + (int64_t)p * d + layers[l].offset;"),
    "delta_ignores_pair_stride": ("const int32_t *sel_i = idx + (int64_t)p * stride_k + out;",
                                  "const int32_t *sel_i = idx + (int64_t)p * k + out;"),
    "model_no_out_advance": ("    out += k;\n  }\n  return 0;\n}\n\n/*\n * Algorithm 1 lines 8-9",
                             "  }\n  return 0;\n}\n\n/*\n * Algorithm 1 lines 8-9"),
}

PIN_FUNCS = [getattr(pins, n) for n in dir(pins) if n.startswith("test_")]


def _run_all_pins(lib):
    """Names of the pins that fail with this library."""
    failed = []
    for f in PIN_FUNCS:
        marks = [m for m in getattr(f, "pytestmark", []) if m.name == "parametrize"]
        if marks:
            names = [n.strip() for n in marks[0].args[0].split(",")]
            calls = [dict(zip(names, v if isinstance(v, tuple) else (v,))) for v in marks[0].args[1]]
        else:
            calls = [{}]
        for kw in calls:
            try:
                f(lib, **kw)
            except (AssertionError, ValueError, IndexError):
                failed.append(f.__name__)
                break
    return failed


def test_unmutated_copy_passes_every_pin():
    assert _run_all_pins(oracle_pkg.OracleLib()) == []


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name):
    old, new = MUTANTS[name]
    src = open(SRC).read()
    if name == "global_indices":
        new = "out_idx[n] = (int32_t)(i + 1);"
    assert src.count(old) >= 1, "mutation site not found: %s" % name      # the first occurrence is mutated
    with tempfile.TemporaryDirectory() as tmp:
        c = os.path.join(tmp, "mutant.c")
        so = os.path.join(tmp, "mutant.so")
        open(c, "w").write(src.replace(old, new, 1))
        subprocess.check_call(["gcc", *oracle_pkg.CFLAGS, "-o", so, c, "-lm"])
        failed = _run_all_pins(oracle_pkg.OracleLib(so))
    assert failed, "no pin notices mutant %s" % name
