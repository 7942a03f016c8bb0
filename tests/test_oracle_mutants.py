"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C source (a dropped term, a
wrong sign or index, a swapped operand), builds it, and runs the pin tests against that copy: they must fail.
CPU only; nothing here touches the GPU path."""
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "npd_oracle.c")

# (name, text in npd_oracle.c, replacement, pin tests that must notice: a -k expression)
MUTANTS = [
    ("lse_drops_max", "return mx + log(z);", "return log(z);", "lse or nll"),
    ("nll_label_index", "return logsumexp(o, V) - o[label];", "return logsumexp(o, V) - o[0];", "nll"),
    ("kl_direction", "if (p_t > 0.0) acc += p_t * (logp_t - logp_s);\n  }\n  if (kd) *kd = acc;\n  if (grad) {\n    for (int64_t c = 0; c < V; ++c) {\n      const double p_s = exp(a[c] - lse_a);",
     "if (p_t > 0.0) acc += p_t * (logp_s - logp_t);\n  }\n  if (kd) *kd = acc;\n  if (grad) {\n    for (int64_t c = 0; c < V; ++c) {\n      const double p_s = exp(a[c] - lse_a);", "kl_"),
    ("teacher_without_tau", "for (int64_t c = 0; c < V; ++c) b[c] = t[c] / tau;\n  const double lse_a = logsumexp(a, V);\n  const double lse_b = logsumexp(b, V);\n  double acc = 0.0;\n  for (int64_t c = 0; c < V; ++c) {\n    const double logp_t = b[c] - lse_b;",
     "for (int64_t c = 0; c < V; ++c) b[c] = t[c];\n  const double lse_a = logsumexp(a, V);\n  const double lse_b = logsumexp(b, V);\n  double acc = 0.0;\n  for (int64_t c = 0; c < V; ++c) {\n    const double logp_t = b[c] - lse_b;", "temperature or library_kl"),
    ("dense_grad_sign", "grad[c] = grad_scale * (1.0 / tau) * (p_s - p_t);", "grad[c] = grad_scale * (1.0 / tau) * (p_t - p_s);", "grad_dense"),
    ("dense_grad_tau_squared", "grad[c] = grad_scale * (1.0 / tau) * (p_s - p_t);", "grad[c] = grad_scale * (1.0 / tau) * (1.0 / tau) * (p_s - p_t);", "grad_dense or temperature"),
    ("topk_student_index", "const double logp_s = a[idx[j]] - lse_a;", "const double logp_s = a[j] - lse_a;", "topk"),
    ("topk_grad_support_sign", "grad[idx[j]] -= grad_scale * (1.0 / tau) * exp(b[j] - lse_b);", "grad[idx[j]] += grad_scale * (1.0 / tau) * exp(b[j] - lse_b);", "grad_topk"),
    ("ce_grad_onehot", "(exp(s[c] - lse) - (c == label ? 1.0 : 0.0))", "(exp(s[c] - lse) + (c == label ? 1.0 : 0.0))", "composite"),
    ("segment_range_off_by_one", "for (int64_t p = cu[i]; p < cu[i + 1]; ++p) {", "for (int64_t p = cu[i] + 1; p < cu[i + 1]; ++p) {", "segment or packing"),
    ("segment_ignores_mask", "      if (mask[p]) {\n        acc += x[p];", "      if (1) {\n        acc += x[p];", "segment or packing"),
    ("delta_direction", "d = it - is;", "d = is - it;", "delta_ifd"),
    ("ifd_inverted", "is = mean_nll_student[ic] / mean_nll_student[iu];", "is = mean_nll_student[iu] / mean_nll_student[ic];", "delta_ifd"),
    ("zone_open_interval", "else if (d32 > (float)hi)", "else if (d32 >= (float)hi)", "delta_ifd"),
    ("ifd_accepts_infinite_mean_loss", "if (ok_counts && ok_means && mean_nll_student[iu] != 0.0", "if (ok_counts && mean_nll_student[iu] != 0.0", "delta_ifd"),
    ("ifd_zone_of_a_non_finite_delta", "if (isfinite(is) && isfinite(it) && isfinite(d)) {", "if (1) {", "delta_ifd"),
    ("ppl_without_exp", "ppl[i] = seg_count[i] > 0 ? exp(mean_nll[i]) : 0.0;", "ppl[i] = seg_count[i] > 0 ? mean_nll[i] : 0.0;", "perplexity"),
    ("policy_lag_mean_of_means", "const double mean = n_total > 0 ? total / (double)n_total : 0.0;", "double mm = 0.0; int32_t ns = 0; for (int32_t i = 0; i < S; ++i) if (seg_count[i] > 0) { mm += seg_mean[i]; ns += 1; }\n  const double mean = ns > 0 ? mm / ns : 0.0;", "policy_lag"),
    ("policy_lag_open_bound", "return !((float)mean <= (float)epsilon);", "return !((float)mean < (float)epsilon);", "policy_lag"),
    ("policy_lag_counts_unscored", "      if (mask[q]) {\n        acc += kl_tok[q];", "      if (1) {\n        acc += kl_tok[q];", "policy_lag"),
    ("teacher_topk_tie_rule", "(best < 0 || row[c] > row[best])", "(best < 0 || row[c] >= row[best])", "teacher_topk"),
    ("reverse_kl_swapped", "if (p_s > 0.0) acc += p_s * (logp_s - logp_t);\n      u[c] = p_s > 0.0 ? logp_s - logp_t + 1.0 : 0.0;", "if (p_s > 0.0) acc += p_s * (logp_t - logp_s);\n      u[c] = p_s > 0.0 ? logp_t - logp_s + 1.0 : 0.0;", "divergence"),
    ("reverse_kl_zero_probability_entry", "u[c] = p_s > 0.0 ? logp_s - logp_t + 1.0 : 0.0;", "u[c] = logp_s - logp_t + 1.0;", "minus_infinity"),
    ("forward_kl_zero_probability_term", "if (p_t > 0.0) acc += p_t * (logp_t - logp_s);\n  }\n  if (kd) *kd = acc;\n  if (grad) {\n    for (int64_t c = 0; c < V; ++c) {", "acc += p_t * (logp_t - logp_s);\n  }\n  if (kd) *kd = acc;\n  if (grad) {\n    for (int64_t c = 0; c < V; ++c) {", "minus_infinity"),
    ("skew_weights_swapped", "const double m = alpha * p_t + (1.0 - alpha) * p_s;\n      if (p_t > 0.0)", "const double m = (1.0 - alpha) * p_t + alpha * p_s;\n      if (p_t > 0.0)", "divergence"),
    ("divergence_grad_without_mean", "grad[c] = grad_scale * (1.0 / tau) * exp(a[c] - lse_a) * (u[c] - ubar);", "grad[c] = grad_scale * (1.0 / tau) * exp(a[c] - lse_a) * u[c];", "divergence"),
]


def _run_pins(lib, expr):
    env = dict(os.environ, NPD_ORACLE_LIB=lib)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-k", expr, "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True,
                          timeout=600)


@pytest.mark.parametrize("name,old,new,expr", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_the_pins(name, old, new, expr):
    sys.path.insert(0, ROOT)
    from oracle import build as oracle_build
    text = open(SRC).read()
    assert text.count(old) == 1, f"{name}: the text to replace must occur exactly once in the oracle"
    with tempfile.TemporaryDirectory(prefix="npd_mutant_") as tmp:
        src, lib = os.path.join(tmp, "npd_oracle.c"), os.path.join(tmp, "libmutant.so")
        with open(src, "w") as f:
            f.write(text.replace(old, new))
        oracle_build.compile_source(src, lib)
        r = _run_pins(lib, expr)
        assert r.returncode == 1, f"{name}: the pins did not notice\n{r.stdout[-2000:]}"
        assert " failed" in r.stdout


def test_the_unmodified_oracle_passes_through_the_same_route():
    sys.path.insert(0, ROOT)
    from oracle import build as oracle_build
    with tempfile.TemporaryDirectory(prefix="npd_mutant_") as tmp:
        lib = oracle_build.compile_source(SRC, os.path.join(tmp, "libsame.so"))
        r = _run_pins(lib, "kl_ or grad_dense or delta_ifd")
        assert r.returncode == 0, r.stdout[-2000:]
