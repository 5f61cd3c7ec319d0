"""Plants one plausible mistake at a time in a copy of the oracle's source (on
the CPU, in a temporary directory) and checks that the pin list catches it.
This is a test of the pins' strength, not of the oracle."""
import os
import subprocess

import pytest

import oracle
from oracle_pins import ALL_PINS

# (name, text in oracle.c, replacement)
MUTANTS = [
    ("dropped_bias", "z[n] = (b ? (double)b[n] : 0.0) + acc;", "z[n] = acc;"),
    ("transposed_W", "const float *w = W + (size_t)n * (size_t)K;\n        double acc = 0.0;\n"
                     "        for (int64_t k = 0; k < K; ++k)\n            acc += (double)x[k] * (double)w[k];",
                     "double acc = 0.0;\n        for (int64_t k = 0; k < K; ++k)\n"
                     "            acc += (double)x[k] * (double)W[(size_t)k * (size_t)N + n];"),
    ("k_off_by_one", "for (int64_t k = 0; k < K; ++k)\n            acc +=", "for (int64_t k = 1; k < K; ++k)\n            acc +="),
    ("erf_sign", "return 0.5 * z * erfc(-z / sqrt(2.0));", "return 0.5 * z * erfc(z / sqrt(2.0));"),
    ("erf_no_sqrt2", "erfc(-z / sqrt(2.0))", "erfc(-z / 2.0)"),
    ("gelu_tanh_form", "return 0.5 * z * erfc(-z / sqrt(2.0));",
     "return 0.5 * z * (1.0 + tanh(0.7978845608028654 * (z + 0.044715 * z * z * z)));"),
    ("unbiased_variance", "const double var = q / (double)N;", "const double var = q / (double)(N - 1);"),
    ("eps_outside_sqrt", "const double denom = sqrt(var + eps);", "const double denom = sqrt(var) + eps;"),
    ("eps_dropped", "const double denom = sqrt(var + eps);", "const double denom = sqrt(var);"),
    ("mean_not_removed", "y[n] = (g[n] - mu) / denom * ga + be;", "y[n] = g[n] / denom * ga + be;"),
    ("gamma_beta_swapped", "y[n] = (g[n] - mu) / denom * ga + be;", "y[n] = (g[n] - mu) / denom * be + ga;"),
    ("beta_dropped", "y[n] = (g[n] - mu) / denom * ga + be;", "y[n] = (g[n] - mu) / denom * ga;"),
    ("row_index", "const int64_t m = rows ? rows[r] : r;", "const int64_t m = r;"),
    ("rowmean_subtract_dropped", "acc += z[n] - (s ? (double)s[n] : 0.0);", "acc += z[n];"),
    ("rowmean_sum_not_mean", "const double g = oracle_gelu(acc / (double)N);", "const double g = oracle_gelu(acc);"),
    ("rowmean_no_residual", "Out[(size_t)r * (size_t)K + k] = (double)x[k] + g;", "Out[(size_t)r * (size_t)K + k] = g;"),
    ("rowmean_gelu_dropped", "const double g = oracle_gelu(acc / (double)N);", "const double g = acc / (double)N;"),
    ("xent_max_not_removed", "se += exp((double)row[c] - mx);", "se += exp((double)row[c]);"),
    ("xent_max_skips_last", "for (int64_t c = 1; c < C; ++c)\n            if ((double)row[c] > mx)",
     "for (int64_t c = 1; c < C - 1; ++c)\n            if ((double)row[c] > mx)"),
    ("xent_max_not_added_back", "loss[r] = mx + log(se) - (double)row[t[r]];", "loss[r] = log(se) - (double)row[t[r]];"),
    ("xent_pick_from_row_index", "loss[r] = mx + log(se) - (double)row[t[r]];",
     "loss[r] = mx + log(se) - (double)row[r % C];"),
    ("xent_sign", "loss[r] = mx + log(se) - (double)row[t[r]];", "loss[r] = (double)row[t[r]] - mx - log(se);"),
    ("xent_log2", "loss[r] = mx + log(se) - (double)row[t[r]];", "loss[r] = mx + log2(se) - (double)row[t[r]];"),
    ("xent_mean_over_classes", "*mean_loss = acc / (double)B;", "*mean_loss = acc / (double)C;"),
    ("xent_target_bound", "if (t[r] < 0 || t[r] >= C)", "if (t[r] < 0 || t[r] > C)"),
    ("bf16_truncates", "const double r = nearbyint(q);", "const double r = trunc(q);"),
    ("bf16_7bits", "ldexp(x, 7 - e)", "ldexp(x, 6 - e)"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, old, new):
    src = open(oracle.SOURCE).read()
    assert src.count(old) >= 1, "mutation site not found: the oracle's text changed, update this test"
    mutated = src.replace(old, new, 1)
    if name == "bf16_7bits":
        mutated = mutated.replace("ldexp(r, e - 7)", "ldexp(r, e - 6)")
    c = tmp_path / "oracle_mutant.c"
    so = tmp_path / ("liboracle_%s.so" % name)
    c.write_text(mutated)
    subprocess.check_call(["gcc", *oracle.CFLAGS, "-o", str(so), str(c), "-lm"])
    orc = oracle.Oracle(str(so))
    caught = []
    for pin in ALL_PINS:
        try:
            pin(orc)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, "no pin noticed mutant %s" % name
