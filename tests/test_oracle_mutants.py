"""Each plausible mistake, planted in a copy of the oracle's source on the CPU, must fail a pin.

This checks the pins, not the oracle: a pin suite that lets a dropped term, a wrong sign, a
wrong index or a transposed operand through would not be pinning anything.
"""
import os
import subprocess

import pytest

import oracle
import oracle_pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "sr_oracle.c")

# (name, text in sr_oracle.c, replacement)
MUTANTS = [
    ("threshold_not_strict", "L > 0 && S > tau", "L > 0 && S >= tau"),
    ("threshold_reversed", "L > 0 && S > tau", "L > 0 && S < tau"),
    ("group_mean_dropped", "S /= (double)r;", ""),
    ("cosine_without_key_norm", "double den = nq * nk;", "double den = nq;"),
    ("cosine_without_query_norm", "double den = nq * nk;", "double den = nk;"),
    ("cubic_drops_quadratic", "t[1] * x * x +", ""),
    ("cubic_coefficients_reversed", "t[0] * x * x * x + t[1] * x * x + t[2] * x + t[3]",
     "t[3] * x * x * x + t[2] * x * x + t[1] * x + t[0]"),
    ("length_not_normalised", "(double)L / c->len_norm", "(double)L"),
    ("scale_dropped", "s *= scale;", ""),
    ("default_scale_is_one_over_d", "1.0 / sqrt((double)c->head_dim)", "1.0 / (double)c->head_dim"),
    ("key_row_off_by_one", "const uint16_t* kr = K + (size_t)t * D;",
     "const uint16_t* kr = K + (size_t)(t > 0 ? t - 1 : 0) * D;"),
    ("value_row_uses_key", "const uint16_t* vr = V + (size_t)t * D;", "const uint16_t* vr = K + (size_t)t * D;"),
    ("softmax_not_normalised", "double u = (L > 0) ? o[d] / l : 0.0;", "double u = (L > 0) ? o[d] : 0.0;"),
    ("group_index_interleaved", "const int b = bh / Hq, h = bh % Hq, g = h / r;\n      const int32_t L = clamp_len(seq_lens[b], Lmax);\n      const int skip",
     "const int b = bh / Hq, h = bh % Hq, g = h % Hkv;\n      const int32_t L = clamp_len(seq_lens[b], Lmax);\n      const int skip"),
    ("sink_group_not_zeroed", "orow[d] = skip ? 0.0 : u;", "orow[d] = u;"),
    ("merge_ignores_chunk_max", "double w = exp(pm[j] - M);", "double w = 1.0;"),
    ("merge_denominator_unweighted", "den += w * pl[j];", "den += pl[j];"),
    ("alpha0_is_last_token", "exp(z[0] - m) / l", "exp(z[L - 1] - m) / l"),
    ("lse_drops_max", "m + log(l)", "log(l)"),
    ("zero_length_still_routed", "c->routing_enabled && L > 0 &&", "c->routing_enabled &&"),
    ("anchor_is_last_row", ": k_cache + ((size_t)b * Hkv + g) * (size_t)c->max_seq_len * D;",
     ": k_cache + ((size_t)b * Hkv + g) * (size_t)c->max_seq_len * D + (size_t)(L > 0 ? L - 1 : 0) * D;"),
    ("separate_anchor_ignored", "const uint16_t* k0 = k0_rows ? k0_rows + ((size_t)b * Hkv + g) * D",
     "const uint16_t* k0 = (0 && k0_rows) ? k0_rows + ((size_t)b * Hkv + g) * D"),
    ("page_row_ignores_offset", "* page_tokens + (t % page_tokens)) * D;", "* page_tokens) * D;"),
    ("page_group_stride_wrong", "const uint16_t* src = pages + (((size_t)page * Hkv + g) * page_tokens",
     "const uint16_t* src = pages + (((size_t)page + (size_t)g * n_pages) * page_tokens"),
    ("page_table_row_stride_wrong", "int32_t page = table[(size_t)b * pages_per_seq + j];", "int32_t page = table[(size_t)b + j];"),
    ("concentration_max_counts_token0", "for (int32_t t = 1; t < L; ++t) {\n        if (w[t] > biggest)",
     "for (int32_t t = 0; t < L; ++t) {\n        if (w[t] > biggest)"),
    ("concentration_mean_over_all_tokens", "rest / (double)(L - 1)", "rest / (double)L"),
    ("concentration_not_normalised", "for (int32_t t = 0; t < L; ++t) w[t] /= total;", ""),
    ("concentration_rest_not_renormalised", "for (int d = 0; d < D; ++d) orow[d] /= rest;", ""),
    ("concentration_scale_dropped", "w[t] = s * scale;", "w[t] = s;"),
    ("negative_length_not_clamped", "if (L < 0) return 0;", ""),
    ("overlong_length_not_clamped_for_tau", "int32_t L = clamp_len(seq_lens[b], c->max_seq_len);\n    double tau = tau_of(c, L);",
     "int32_t L = clamp_len(seq_lens[b], c->max_seq_len);\n    double tau = tau_of(c, seq_lens[b]);"),
    ("nan_denominator_not_zeroed", "if (!(den > 0.0)) return 0.0;", "if (den == 0.0) return 0.0;"),
    ("nan_cached_norm_used", "nk = anchor_norm >= 0.0 ? anchor_norm : sqrt(nk);", "nk = !(anchor_norm < 0.0) ? anchor_norm : sqrt(nk);"),
    ("separate_anchor_wrong_group", "k0_rows + ((size_t)b * Hkv + g) * D", "k0_rows + ((size_t)b * Hkv) * D"),
]


@pytest.fixture(scope="module")
def source():
    return open(SRC).read()


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(name, old, new, source, tmp_path):
    assert source.count(old) >= 1, "mutation site not found: %s" % name
    mutated = source.replace(old, new, 1)
    c = tmp_path / "mut.c"
    so = tmp_path / ("mut_%s.so" % name)
    c.write_text(mutated)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
                    str(c), "-o", str(so), "-lm"], check=True)
    caught = []
    for pin in oracle_pins.ALL_PINS:
        try:
            pin(str(so))
        except (AssertionError, RuntimeError):      # a pin fails, or the broken oracle itself reports an error
            caught.append(pin.__name__)
    assert caught, "no pin notices the planted mistake '%s'" % name
