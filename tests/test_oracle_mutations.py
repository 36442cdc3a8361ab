"""The pins must notice a plausible mistake anywhere in the oracle.

Each case plants one mistake in a COPY of oracle/turbo_oracle.c (a dropped term, a wrong sign or index, a
transposed operand), compiles it on the CPU, and runs the pin suite against it in a subprocess: the suite has to fail.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "turbo_oracle.c")

MUTATIONS = [
    ("mask_is_scaled", "double z = scale * s[k] + (a ? a[k] : 0.0);", "double z = scale * (s[k] + (a ? a[k] : 0.0));"),
    ("mask_subtracted", "double z = scale * s[k] + (a ? a[k] : 0.0);", "double z = scale * s[k] - (a ? a[k] : 0.0);"),
    ("scale_dropped", "double z = scale * s[k] + (a ? a[k] : 0.0);", "double z = s[k] + (a ? a[k] : 0.0);"),
    ("mask_strides_swapped", "mask + b * mask_stride_b + q * mask_stride_q", "mask + q * mask_stride_b + b * mask_stride_q"),
    ("query_index_wrong", "long long q = row % Sq;", "long long q = row % H;"),
    ("batch_index_wrong", "long long b = row / ((long long)H * Sq);", "long long b = row / Sq;"),
    ("no_max_shift", "y[k] = exp(y[k] - m);", "y[k] = exp(y[k]);"),
    ("max_starts_at_zero", "double m = -INFINITY;", "double m = 0.0;"),
    ("not_normalised", "for (int k = 0; k < Sk; ++k) y[k] /= l;", ""),
    ("sample_variance", "double var = ss / hidden;", "double var = ss / (hidden - 1);"),
    ("eps_outside_sqrt", "double inv = 1.0 / sqrt(var + eps);", "double inv = 1.0 / (sqrt(var) + eps);"),
    ("bias_dropped", "double t = xr[j] + (bias ? bias[j] : 0.0) + (rr ? rr[j] : 0.0);", "double t = xr[j] + (rr ? rr[j] : 0.0);"),
    ("residual_dropped", "double t = xr[j] + (bias ? bias[j] : 0.0) + (rr ? rr[j] : 0.0);", "double t = xr[j] + (bias ? bias[j] : 0.0);"),
    ("residual_subtracted", "(bias ? bias[j] : 0.0) + (rr ? rr[j] : 0.0);", "(bias ? bias[j] : 0.0) - (rr ? rr[j] : 0.0);"),
    ("gamma_beta_swapped", "(o[j] - mu) * inv * gamma[j] + beta[j];", "(o[j] - mu) * inv * beta[j] + gamma[j];"),
    ("mean_not_removed_in_variance", "double d = o[j] - mu;\n            ss += d * d;", "double d = o[j];\n            ss += d * d;"),
    ("mean_not_removed_in_output", "o[j] = (o[j] - mu) * inv * gamma[j] + beta[j];", "o[j] = o[j] * inv * gamma[j] + beta[j];"),
    ("residual_row_stride_wrong", "residual ? residual + r * hidden : NULL;", "residual ? residual + r : NULL;"),
    ("eq1_second_form_wrong", "return s2 / n - mu * mu;", "return s2 / n - mu;"),
    ("welford_update_wrong", "m2 += d * (x[i] - mean);", "m2 += d * d;"),
    ("chan_cross_term_dropped", "*m2 = m2_a + m2_b + d * d * (na * nb / nt);", "*m2 = m2_a + m2_b;"),
    ("gelu_erfc_sign", "y = t * 0.5 * erfc(-t * 0.7071067811865476);", "y = t * 0.5 * erfc(t * 0.7071067811865476);"),
    ("gelu_missing_half", "y = t * 0.5 * erfc(-t * 0.7071067811865476);", "y = t * erfc(-t * 0.7071067811865476);"),
    ("gelu_tanh_cubic_constant", "0.044715 * t * t * t", "0.44715 * t * t * t"),
    ("gelu_tanh_square_not_cube", "0.044715 * t * t * t", "0.044715 * t * t"),
    ("gelu_bias_dropped", "double t = x[r * hidden + j] + (bias ? bias[j] : 0.0);", "double t = x[r * hidden + j];"),
    ("split_source_order", "((((long long)b * S + s) * n_split + k) * H + h) * D + d;", "((((long long)b * S + s) * H + h) * n_split + k) * D + d;"),
    ("split_dest_heads_and_sequence_swapped", "((((long long)k * B + b) * H + h) * S + s) * D + d;", "((((long long)k * B + b) * S + s) * H + h) * D + d;"),
    ("split_bias_ignores_split_index", "bias[((long long)k * H + h) * D + d]", "bias[((long long)h) * D + d]"),
    ("varlen_softmax_reads_one_key_too_many", "for (int k = 0; k < kl; ++k) {\n                    y[k] = exp(scale * s[k] - m);", "for (int k = 0; k <= kl && k < Sk; ++k) {\n                    y[k] = exp(scale * s[k] - m);"),
    ("varlen_softmax_tail_not_zeroed", "for (int k = kl; k < Sk; ++k) y[k] = 0.0;", "for (int k = kl; k < Sk; ++k) y[k] = s[k];"),
    ("varlen_softmax_ignores_query_lengths", "int active = kl > 0 && (q_len == NULL || q < q_len[b]);", "int active = kl > 0;"),
    ("varlen_layernorm_off_by_one_row", "if (s < len[b])\n                oracle_add_bias_layernorm(", "if (s <= len[b])\n                oracle_add_bias_layernorm("),
    ("packed_request_offset_forgets_the_heads", "base += (long long)H * n * n;", "base += n * n;"),
    ("packed_row_stride_wrong", "const double *s = scores + base + (h * n + q) * n;", "const double *s = scores + base + (h * n + q) * (n - 1);"),
    ("packed_scale_dropped_in_exp", "y[k] = exp(scale * s[k] - m);\n                    l += y[k];\n                }\n                for (long long k = 0; k < n; ++k) y[k] /= l;",
     "y[k] = exp(s[k] - m);\n                    l += y[k];\n                }\n                for (long long k = 0; k < n; ++k) y[k] /= l;"),
    ("causal_diagonal_off_by_one", "int visible = q + (Sk - Sq) + 1;", "int visible = q + (Sk - Sq);"),
    ("causal_offset_sign", "int visible = q + (Sk - Sq) + 1;", "int visible = q - (Sk - Sq) + 1;"),
    ("causal_ignores_key_lengths", "if (k_len != NULL && k_len[b] < visible) visible = k_len[b];", ""),
    ("merge_is_a_copy", "out[(((long long)b * S + s) * H + h) * D + d] = x[(((long long)b * H + h) * S + s) * D + d];",
     "out[(((long long)b * S + s) * H + h) * D + d] = x[(((long long)b * S + s) * H + h) * D + d];"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for {name} not found exactly once"
    mutated = tmp_path / "mutant.c"
    mutated.write_text(text.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-o", str(lib),
                           str(mutated), "-lm"])
    env = dict(os.environ, TURBO_ORACLE_LIB=str(lib))
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                          os.path.join(ROOT, "tests", "test_oracle_pins_elementwise.py"),
                          os.path.join(ROOT, "tests", "test_oracle_pins_varlen.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], env=env, cwd=ROOT, capture_output=True, text=True)
    assert res.returncode != 0, f"the pins did not notice the planted mistake '{name}'"
    assert "failed" in res.stdout or "error" in res.stdout.lower()
