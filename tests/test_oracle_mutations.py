"""The pins must bite: each plausible mistake planted in a COPY of the oracle source
(on the CPU, never in the GPU code) has to make at least one pin test fail."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "gac_oracle.cpp")

# (name, text in the oracle source, replacement)
MUTATIONS = [
    ("eps_under_sqrt", "s_gd / (std::sqrt(s_gg * s_dd) + eps)", "s_gd / std::sqrt(s_gg * s_dd + eps)"),
    ("dropped_eps", "s_gd / (std::sqrt(s_gg * s_dd) + eps)", "s_gd / std::sqrt(s_gg * s_dd)"),
    ("safe_exclusive", "if (a <= c_low) {", "if (a < c_low) {"),
    ("skip_exclusive", "} else if (a >= c_high) {", "} else if (a > c_high) {"),
    ("signed_threshold", "const double a = std::fabs(c);", "const double a = c;"),
    ("alpha_inverted", "out->alpha = c_low / a;", "out->alpha = a / c_low;"),
    ("norm_of_g_for_u", "const double norm_d = std::sqrt(sums[2]);", "const double norm_d = std::sqrt(sums[1]);"),
    ("rank_one_wrong_norm", "(alpha - beta) * (sums[0] / sums[2])", "(alpha - beta) * (sums[0] / sums[1])"),
    ("rank_one_sign", "(alpha - beta) * (sums[0] / sums[2])", "(beta - alpha) * (sums[0] / sums[2])"),
    ("perp_dropped", "g_out[i] = alpha * g_par + beta * g_perp;", "g_out[i] = alpha * g_par;"),
    ("sums_swapped", "out[1] = s_gg;\n  out[2] = s_dd;", "out[1] = s_dd;\n  out[2] = s_gg;"),
    ("state_not_updated_on_skip", "if (!dec.nonfinite) {", "if (!dec.nonfinite && dec.regime != ORACLE_SKIP) {"),
    ("bf16_low_half", "static_cast<uint32_t>(h) << 16;", "static_cast<uint32_t>(h) << 15;"),
    ("adam_no_bias_correction2", "std::sqrt(vi / bc2)", "std::sqrt(vi)"),
    ("clip_eps_dropped", "double scale = max_norm / (norm + 1e-6);", "double scale = max_norm / norm;"),
    ("clip_always_scales", "if (!(scale < 1.0)) return 1.0;", "if (false) return 1.0;"),
    ("quantile_nearest_rank", "out[0] = a[lo] + (a[hi] - a[lo]) * (pos - static_cast<double>(lo));", "out[0] = a[hi];"),
    ("stats_ignore_burn_in", "for (int64_t t = burn_in; t < n; ++t)", "for (int64_t t = 0; t < n; ++t)"),
    ("stats_strict_threshold", "inside += (x <= c_low) ? 1 : 0;", "inside += (x < c_low) ? 1 : 0;"),
    ("sweep_safe_exclusive", "if (mag <= c_low) regime = ORACLE_SAFE;", "if (mag < c_low) regime = ORACLE_SAFE;"),
    ("sweep_skip_exclusive", "else if (mag >= c_high) regime = ORACLE_SKIP;", "else if (mag > c_high) regime = ORACLE_SKIP;"),
    ("sweep_signed", "const double mag = std::fabs(c[step - 1]);", "const double mag = c[step - 1];"),
    ("sweep_burn_in_off_by_one", "for (int64_t step = burn_in + 1; step <= n; ++step) {", "for (int64_t step = burn_in; step <= n; ++step) {"),
    ("sweep_counts_nonfinite_steps", "if (std::isnan(mag)) continue;", ""),
    ("stats_count_nonfinite_steps", "if (!std::isnan(c[t])) a.push_back(std::fabs(c[t]));", "a.push_back(std::fabs(c[t]));"),
    ("adam_coupled_decay", "pi = pi - lr * weight_decay * pi;", "pi = pi - weight_decay * pi;"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation anchor for {name} not unique in the oracle source"
    mutated = tmp_path / "gac_oracle_mutated.cpp"
    mutated.write_text(text.replace(old, new))
    env = dict(os.environ, GAC_ORACLE_SRC=str(mutated), GAC_ORACLE_LIB=str(tmp_path / "libmut.so"))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 1, f"mutation {name} survived the pins:\n{r.stdout[-2000:]}"
