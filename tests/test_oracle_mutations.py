"""Do the pins bite?  Plausible mistakes are planted in COPIES of oracle/kunlun_oracle.c (on the
CPU; the GPU library is not involved), each copy is compiled and put through the pin battery
of tests/test_oracle_pins.py, and every one of them must be caught by at least one pin."""
import os
import subprocess

import pytest

from tests import test_oracle_pins as pins
from tests import test_oracle_sumkron_pins as kpins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "kunlun_oracle.c")

# (name, text to find, replacement, which occurrence)
MUTANTS = [
    ("scores_not_scaled", "s[j] = scale * dot;", "s[j] = dot;", 0),
    ("softmax_exponent_sign", "const double p = exp(s[j] - m) / z;", "const double p = exp(m - s[j]) / z;", 0),
    ("lse_without_max", "= m + log(z);", "= log(z);", 0),
    ("window_left_off_by_one", "*lo = i - left;", "*lo = i - left + 1;", 0),
    ("window_right_off_by_one", "*hi = i + right;", "*hi = i + right + 1 < n_kv ? i + right + 1 : n_kv - 1;", 0),
    ("value_row_of_wrong_head", "const double* vj = v + (k0 + j) * hd + (int64_t)h * d;",
     "const double* vj = v + (k0 + j) * hd;", 1),
    ("empty_history_lse_zero", "lse[(int64_t)h * total_q + q0 + i] = -INFINITY;", "lse[(int64_t)h * total_q + q0 + i] = 0.0;", 0),
    ("silu_sign", "case ACT_SILU: return x / (1.0 + exp(-x));", "case ACT_SILU: return x / (1.0 + exp(x));", 0),
    ("gelu_tanh_coefficient", "double u = SQRT_2_OVER_PI * (x + 0.044715 * x * x * x);\n        return 0.5 * x",
     "double u = SQRT_2_OVER_PI * (x + 0.44715 * x * x * x);\n        return 0.5 * x", 0),
    ("gelu_derivative_drops_pdf_term", "return cdf + x * pdf;", "return cdf;", 0),
    ("gelu_poly_coefficient_sign", "9.2376422360e-03, -9.1053389233e-04,", "9.2376422360e-03, 9.1053389233e-04,", 0),
    ("gelu_poly_not_clamped", "(x > GELU_POLY_C ? GELU_POLY_C : x);", "(x > GELU_POLY_C ? x : x);", 0),
    ("gelu_poly_slope_drops_chain_term", "? q + 2.0 * u * dq : 0.0;", "? q : 0.0;", 0),
    ("gelu_poly_slope_not_zero_outside", "(x > -GELU_POLY_C && x < GELU_POLY_C) ? q + 2.0 * u * dq : 0.0;",
     "q + 2.0 * u * dq;", 0),
    ("backward_scores_not_scaled", "s[j] = scale * dot;", "s[j] = dot;", 1),
    ("softmax_backward_drops_delta", "p[j] * (dp[j] - delta) * scale", "p[j] * dp[j] * scale", 0),
    ("activation_backward_drops_scale", ": dp[j] * act_deriv(a, s[j]) * scale;", ": dp[j] * act_deriv(a, s[j]);", 0),
    ("dq_uses_queries", "dq[qrow + c] += ds * k[krow + c];", "dq[qrow + c] += ds * q[qrow + c];", 0),
    ("dk_uses_keys", "dk[krow + c] += ds * q[qrow + c];", "dk[krow + c] += ds * k[krow + c];", 0),
    ("dv_uses_ds", "dv[krow + c] += p[j] * d_o[qrow + c];", "dv[krow + c] += ds * d_o[qrow + c];", 0),
    ("dp_uses_keys", "dpj += d_o[qrow + c] * v[krow + c];", "dpj += d_o[qrow + c] * k[krow + c];", 0),
    # SumKronLinear
    ("sumkron_z_not_transposed", "const double zst = z[((int64_t)i * S + s) * T + t];",
     "const double zst = z[((int64_t)i * S + (s % T)) * T + (t % S)];", 0),
    ("sumkron_w_transposed", "const double* wc = w + (int64_t)i * D * D + e;\n                        double inner = 0.0;\n"
     "                        for (int c = 0; c < D; ++c) inner += xr[c] * wc[(int64_t)c * D];",
     "const double* wc = w + (int64_t)i * D * D + (int64_t)e * D;\n                        double inner = 0.0;\n"
     "                        for (int c = 0; c < D; ++c) inner += xr[c] * wc[c];", 0),
    ("sumkron_weight_of_first_term_only", "const double* wc = w + (int64_t)i * D * D + e;", "const double* wc = w + e;", 0),
    ("sumkron_dx_uses_w_transposed", "const double* wr = w + ((int64_t)i * D + c) * D;\n                        double inner = 0.0;\n"
     "                        for (int e = 0; e < D; ++e) inner += dyr[e] * wr[e];",
     "const double* wr = w + (int64_t)i * D * D + c;\n                        double inner = 0.0;\n"
     "                        for (int e = 0; e < D; ++e) inner += dyr[e] * wr[(int64_t)e * D];", 0),
    ("sumkron_dz_drops_batch_sum", "for (int b = 0; b < B; ++b) {\n                    const double* xr = x + ((int64_t)b * S + s) * D;",
     "for (int b = 0; b < 1; ++b) {\n                    const double* xr = x + ((int64_t)b * S + s) * D;", 0),
    ("sumkron_dw_uses_wrong_z_term", "inner += z[((int64_t)i * S + s) * T + t] * dy[((int64_t)b * T + t) * D + e];",
     "inner += z[((int64_t)0 * S + s) * T + t] * dy[((int64_t)b * T + t) * D + e];", 0),
]


def _battery():
    """Pin calls, cheap ones first: (function, kwargs)."""
    calls = []
    for c in pins._golden_cases():
        act, scale, q, k, v, o = c.values
        calls.append((pins.test_hand_worked, dict(act=act, scale=scale, q=q, k=k, v=v, o_expected=o)))
    for x in (-2.5, -0.3, 0.7, 2.0):
        calls.append((pins.test_activation_values_vs_libraries, dict(x=x)))
        for name in ("gelu", "gelu_tanh", "silu"):
            calls.append((pins.test_activation_derivatives_vs_autograd, dict(name=name, x=x)))
    calls.append((pins.test_polynomial_gelu_tracks_gelu_and_has_exact_tails, {}))
    for x in (-4.0, -1.2, 0.4, 3.3):
        calls.append((pins.test_activation_derivatives_vs_autograd, dict(name="gelu_poly", x=x)))
    calls.append((pins.test_lse_consistency, {}))
    calls.append((pins.test_softmax_special_cases, {}))
    calls.append((pins.test_window_special_cases, {}))
    for act in ("softmax", "gelu", "silu", "gelu_tanh"):
        calls.append((pins.test_gdpa_forward_vs_bruteforce, dict(seed=0, act=act)))
    calls.append((pins.test_gdpa_forward_dense_q_and_per_head_activation, {}))
    for window in ((2, 0), (1, 4), (0, 3)):
        calls.append((pins.test_swa_forward_vs_bruteforce, dict(window=window)))
    calls.append((pins.test_dense_equal_lengths_match_library_attention_and_autograd, {}))
    for act in ("gelu", "silu", "identity"):
        calls.append((pins.test_activation_mode_backward_vs_autograd, dict(act=act)))
    for act in ("softmax", "gelu"):
        calls.append((pins.test_gdpa_backward_finite_differences, dict(act=act)))
    calls.append((pins.test_swa_backward_finite_differences, dict(window=(2, 0))))
    calls.append((kpins.test_sumkron_hand_worked, {}))
    calls.append((kpins.test_sumkron_equals_explicit_kronecker_matrix, {}))
    calls.append((kpins.test_sumkron_single_entry_probes, {}))
    calls.append((kpins.test_sumkron_selection_and_separable_cases, {}))
    calls.append((kpins.test_sumkron_backward_finite_differences, {}))
    calls.append((kpins.test_sumkron_backward_vs_autograd, {}))
    return calls


def _first_failing_pin(lib):
    for fn, kw in _battery():
        try:
            fn(lib, **kw)
        except AssertionError:
            return fn.__name__
    return None


def test_unmodified_oracle_passes_the_battery(oracle):
    assert _first_failing_pin(oracle) is None


@pytest.mark.parametrize("name,find,repl,occurrence", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(oracle, tmp_path, name, find, repl, occurrence):
    text = open(SRC).read()
    parts = text.split(find)
    assert len(parts) > occurrence + 1, f"mutation site for {name} not found"
    mutated = find.join(parts[:occurrence + 1]) + repl + find.join(parts[occurrence + 1:])
    src = tmp_path / f"{name}.c"
    lib = tmp_path / f"lib{name}.so"
    src.write_text(mutated)
    subprocess.run(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", str(lib), str(src), "-lm"], check=True)
    caught_by = _first_failing_pin(oracle.OracleLib(str(lib)))
    assert caught_by is not None, f"no pin notices the planted mistake '{name}'"
