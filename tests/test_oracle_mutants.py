"""Shows that the oracle's pins are sharp: each plausible mistake, planted in a copy of the oracle's
source on the CPU, makes tests/test_oracle_pins.py or tests/test_oracle_dgc.py fail."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sidco_oracle.c")

# (name, text in the oracle, replacement)
MUTANTS = [
    ("exp_sign", "return mu * log(1.0 / delta);", "return mu * log(delta);"),
    ("gpd_alpha_sign", "*alpha = 0.5 * (1.0 - q);", "*alpha = 0.5 * (q - 1.0);"),
    ("gpd_sigma_not_squared", "double q = (mu * mu) / var;", "double q = (mu * mu) / sqrt(var);"),
    ("gpd_ratio_transposed", "double q = (mu * mu) / var;", "double q = var / (mu * mu);"),
    ("gpd_beta_minus", "*beta = 0.5 * mu * (q + 1.0);", "*beta = 0.5 * mu * (q - 1.0);"),
    ("gpd_exponent_sign", "expm1(-a * log(delta))", "expm1(a * log(delta))"),
    ("pot_shift_forgotten", "double y = (double)a - (double)eta_prev;", "double y = (double)a;"),
    ("pot_exp_location_dropped", "(double)eta_prev + sidco_oracle_eta_exp(ybar, ratios[m])",
     "sidco_oracle_eta_exp(ybar, ratios[m])"),
    ("pot_gpd_location_dropped", "(double)eta_prev + sidco_oracle_eta_gpd(ybar, yvar, ratios[m])",
     "sidco_oracle_eta_gpd(ybar, yvar, ratios[m])"),
    ("pot_wrong_ratio", "sidco_oracle_eta_exp(ybar, ratios[m])", "sidco_oracle_eta_exp(ybar, ratios[0])"),
    ("select_non_strict", "if (fabsf(acc[j]) > eta) {", "if (fabsf(acc[j]) >= eta) {"),
    ("pot_non_strict", "if (a > eta_prev) {", "if (a >= eta_prev) {"),
    ("variance_bessel", "*yvar = s2 / (double)n - m * m;",
     "*yvar = (s2 / (double)n - m * m) * (double)n / (double)(n > 1 ? n - 1 : 1);"),
    ("second_moment_dropped", "s2 += x * x;", "s2 += x;"),
    ("variance_is_mean_square", "*var = s2 / (double)d - m * m;", "*var = s2 / (double)d;"),
    ("gamma_shape_constant", "24.0 * s", "12.0 * s"),
    ("gamma_lgamma_dropped", "return -b * (log(delta) + lgamma(a));", "return -b * log(delta);"),
    ("gamma_s_sign", "double s = log(mu) - mulog;\n    double a", "double s = mulog - log(mu);\n    double a"),
    ("residual_not_zeroed", "if (residual) residual[j] = 0.0f;", ""),
    ("ec_add_dropped", "volatile float s = g[j] + r[j];", "volatile float s = g[j];"),
    ("schedule_no_root", "pow(delta / delta1, 1.0 / (double)(stages - 1))", "delta / delta1"),
    ("adapt_up_down_swapped", "if (khat_avg > k * (1.0 + eps_h)) M = M - 1;", "if (khat_avg > k * (1.0 + eps_h)) M = M + 1;"),
    ("adapt_low_band_uses_high_eps", "if (khat_avg < k * (1.0 - eps_l)) M = M + 1;",
     "if (khat_avg < k * (1.0 - eps_h)) M = M + 1;"),
    ("adapt_non_strict", "if (khat_avg > k * (1.0 + eps_h)) M = M - 1;", "if (khat_avg >= k * (1.0 + eps_h)) M = M - 1;"),
    ("adapt_no_upper_clamp", "if (M > M_max) M = M_max;", ""),
    ("adapt_no_lower_clamp", "if (M < 1) M = 1;\n    if (M > M_max)", "if (M > M_max)"),
    ("scatter_scale_dropped", "volatile float prod = scale * val[i];", "volatile float prod = val[i];"),
    ("scatter_overwrites", "volatile float sum = dense[j] + prod;", "volatile float sum = prod;"),
    ("scatter_upper_bound_off_by_one", "if (j < 0 || j >= d) {", "if (j < 0 || j > d) {"),
    ("signed_values_lost", "if (val) val[k] = acc[j];", "if (val) val[k] = fabsf(acc[j]);"),
    # the DGC comparator
    ("dgc_generator_shift", "z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;", "z = (z ^ (z >> 29)) * 0x94D049BB133111EBull;"),
    ("dgc_generator_first_output_skipped", "seed + (j + 1u) * 0x9E3779B97F4A7C15ull", "seed + (j + 2u) * 0x9E3779B97F4A7C15ull"),
    ("dgc_index_from_low_bits", "uint64_t u = splitmix64_at(seed, j) >> 32;", "uint64_t u = splitmix64_at(seed, j) & 0xffffffffu;"),
    ("dgc_rank_off_by_one", "uint32_t kappa = keys[k_s - 1];", "uint32_t kappa = keys[k_s];"),
    ("dgc_sorted_ascending", "return (x < y) - (x > y);", "return (x > y) - (x < y);"),
    ("dgc_first_pass_non_strict", "{ return fabsf(x) > eta; }", "{ return fabsf(x) >= eta; }"),
    ("dgc_always_trims_to_k_s", "keep = k;", "keep = k_s;"),
    ("dgc_sample_of_gradient_not_acc", "keys[j] = mag_bits(acc[", "keys[j] = mag_bits(g["),
    ("dgc_residual_kept", "if (r) r[idx[i]] = 0.0f;", ""),
]


def _run_mutant(args):
    name, old, new, tmp = args
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutant {name}: pattern not found in oracle source"
    src = os.path.join(tmp, name + ".c")
    lib = os.path.join(tmp, name + ".so")
    with open(src, "w") as f:
        f.write(text.replace(old, new))
    subprocess.run(["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-o", lib, src, "-lm"],
                   check=True, capture_output=True)
    env = dict(os.environ, SIDCO_ORACLE_LIB=lib)
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_oracle_dgc.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    return name, p.returncode


def test_every_planted_mistake_is_caught(tmp_path):
    jobs = [(n, o, r, str(tmp_path)) for n, o, r in MUTANTS]
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(_run_mutant, jobs))
    survivors = [n for n, rc in results if rc == 0]
    assert not survivors, f"pins did not catch: {survivors}"
    assert all(rc == 1 for _, rc in results), results  # 1 = tests failed (not a collection error)
