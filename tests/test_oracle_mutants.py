"""Do the oracle's pins have teeth?  Each case below plants one plausible mistake in a
copy of the oracle's source (on the CPU; no GPU is involved), builds it, and runs the pin
tests against that build: they must fail.  The unmodified source must pass the same way.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "rmsnorm_oracle.cpp")
PINS = os.path.join(ROOT, "tests", "test_oracle_pins.py")

MUTANTS = {
    "mean_over_n_minus_1": ("const double ms = ss / (double)N;",
                            "const double ms = ss / (double)(N > 1 ? N - 1 : 1);"),
    "eps_outside_the_root": ("1.0 / std::sqrt(ms + eps)", "1.0 / (std::sqrt(ms) + eps)"),
    "missing_root": ("1.0 / std::sqrt(ms + eps)", "1.0 / (ms + eps)"),
    "first_element_dropped": ("double ss = 0.0;\n    for (int64_t j = 0; j < N; ++j) {",
                              "double ss = 0.0;\n    for (int64_t j = 1; j < N; ++j) {"),
    "last_element_dropped": ("double ss = 0.0;\n    for (int64_t j = 0; j < N; ++j) {",
                             "double ss = 0.0;\n    for (int64_t j = 0; j + 1 < N || j == 0; ++j) {"),
    "sum_of_abs_not_squares": ("ss += xv * xv;", "ss += std::fabs(xv);"),
    "weight_shifted_by_one": ("const double v = xv * r * wd[(size_t)j];",
                              "const double v = xv * r * wd[(size_t)((j + 1) % N)];"),
    "weight_indexed_by_row": ("const double v = xv * r * wd[(size_t)j];",
                              "const double v = xv * r * wd[(size_t)(i % N)];"),
    "weight_forgotten": ("const double v = xv * r * wd[(size_t)j];", "const double v = xv * r;"),
    "x_read_transposed": ("const double xv = decode_bits(load_bits(x, i * N + j, dtype), f);\n      const double v",
                          "const double xv = decode_bits(load_bits(x, (i * N + j) % (N * ((i * N + j) / N + 1)) == 0 ? 0 : i * N + (N - 1 - j), dtype), f);\n      const double v"),
    "rounds_through_fp32_first": ("encode_bits(round_to_format(v, f), f)",
                                  "encode_bits(round_to_format((double)(float)v, f), f)"),
    "encode_rounds_through_fp32_first": ("encode_bits(round_to_format(src[k], *f), *f)",
                                         "encode_bits(round_to_format((double)(float)src[k], *f), *f)"),
    "ties_away_from_zero": ("std::nearbyint(std::ldexp(a, f.p - 1 - e))",
                            "std::round(std::ldexp(a, f.p - 1 - e))"),
    "truncates": ("std::nearbyint(std::ldexp(a, f.p - 1 - e))", "std::floor(std::ldexp(a, f.p - 1 - e))"),
    "subnormals_flushed": ("if (e < f.emin) e = f.emin;", "if (e < f.emin) return std::copysign(0.0, v);"),
    "no_overflow_to_infinity": ("if (r > max_finite) return std::copysign(INFINITY, v);",
                                "if (r > max_finite) return std::copysign(max_finite, v);"),
    "fp16_bias_off_by_one": ("constexpr Format kFp16{11, -14, 15, 5};", "constexpr Format kFp16{11, -14, 16, 5};"),
    "bf16_mantissa_width": ("constexpr Format kBf16{8, -126, 127, 8};", "constexpr Format kBf16{7, -126, 127, 8};"),
    "sign_lost": ("return neg ? -v : v;", "return v;"),
    "rstd_squared_input": ("const double r = 1.0 / std::sqrt(ms + eps);",
                           "const double r = 1.0 / std::sqrt(ms * ms + eps);"),
}


SOFTMAX_SRC = os.path.join(ROOT, "oracle", "softmax_oracle.cpp")
SOFTMAX_PINS = os.path.join(ROOT, "tests", "test_softmax_oracle_pins.py")

SOFTMAX_MUTANTS = {
    "no_max_subtraction": ("std::exp(v - m); ", "std::exp(v); "),
    "base_two_exponential": ("std::exp(v - m); ", "std::exp2(v - m); "),
    "first_term_missing_from_the_sum": ("s += e[(size_t)j];", "if (j > 0 || N == 1) s += e[(size_t)j];"),
    "divides_by_the_mean": ("e[(size_t)j] / s;", "e[(size_t)j] / (s / (double)N);"),
    "max_of_absolute_values": ("else if (v > m) m = v;", "else if (std::fabs(v) > m) m = std::fabs(v);"),
    # (no ties-away-from-zero case here: a quotient exp(.)/sum computed in fp64 never lands
    #  exactly on a 16-bit or fp32 tie except for dyadic 1/2^k, which is representable)
    "truncates": ("std::nearbyint(std::ldexp(a, mbits - e))", "std::floor(std::ldexp(a, mbits - e))"),
    "rounds_up": ("std::nearbyint(std::ldexp(a, mbits - e))", "std::ceil(std::ldexp(a, mbits - e))"),
    "subnormals_flushed": ("if (e < f.emin) e = f.emin;", "if (e < f.emin) return sign;"),
    "rounds_through_fp32_first": ("store_bits(y, i * N + j, dtype, narrow(out, f));",
                                  "store_bits(y, i * N + j, dtype, narrow((double)(float)out, f));"),
    "nan_row_not_propagated": ("const double out = has_nan ? std::nan(\"\") : e[(size_t)j] / s;",
                               "const double out = std::isnan(e[(size_t)j]) ? 0.0 : e[(size_t)j] / (std::isnan(s) ? 1.0 : s);"),
}


LAYERNORM_SRC = os.path.join(ROOT, "oracle", "layernorm_oracle.cpp")
LAYERNORM_PINS = os.path.join(ROOT, "tests", "test_layernorm_oracle_pins.py")

LAYERNORM_MUTANTS = {
    "unbiased_variance": ("const double var = spread / static_cast<double>(N);",
                          "const double var = spread / static_cast<double>(N > 1 ? N - 1 : 1);"),
    "second_moment_not_centred": ("      spread += c * c;\n", "      spread += (c + mu) * (c + mu);\n"),
    "mean_not_subtracted_in_output": ("      const double out = c * rstd *", "      const double out = (c + mu) * rstd *"),
    "eps_outside_the_root": ("1.0 / std::sqrt(var + eps)", "1.0 / (std::sqrt(var) + eps)"),
    "missing_root": ("1.0 / std::sqrt(var + eps)", "1.0 / (var + eps)"),
    "mean_over_n_minus_1": ("const double mu = total / static_cast<double>(N);",
                            "const double mu = total / static_cast<double>(N > 1 ? N - 1 : 1);"),
    "bias_forgotten": ("+ bv[static_cast<size_t>(j)];", "+ 0.0 * bv[static_cast<size_t>(j)];"),
    "bias_scaled_by_weight": ("const double out = c * rstd * wv[static_cast<size_t>(j)] + bv[static_cast<size_t>(j)];",
                              "const double out = (c * rstd + bv[static_cast<size_t>(j)]) * wv[static_cast<size_t>(j)];"),
    "weight_shifted_by_one": ("c * rstd * wv[static_cast<size_t>(j)]", "c * rstd * wv[static_cast<size_t>((j + 1) % N)]"),
    "bias_indexed_by_row": ("+ bv[static_cast<size_t>(j)];", "+ bv[static_cast<size_t>(i % N)];"),
    "first_element_missing_from_the_mean": ("    double total = 0.0;\n    for (int64_t j = 0; j < N; ++j) total",
                                            "    double total = 0.0;\n    for (int64_t j = (N > 1 ? 1 : 0); j < N; ++j) total"),
    "rounds_through_fp32_first": ("put_bits(y, i * N + j, dtype, from_double(out, L));",
                                  "put_bits(y, i * N + j, dtype, from_double((double)(float)out, L));"),
    "ties_away_from_zero": ("std::nearbyint(std::ldexp(a, frac_bits - e))", "std::round(std::ldexp(a, frac_bits - e))"),
    "truncates": ("std::nearbyint(std::ldexp(a, frac_bits - e))", "std::floor(std::ldexp(a, frac_bits - e))"),
    "sign_lost": ("return minus ? -v : v;", "return v;"),
}


CE_SRC = os.path.join(ROOT, "oracle", "crossentropy_oracle.cpp")
CE_PINS = os.path.join(ROOT, "tests", "test_crossentropy_oracle_pins.py")

CE_MUTANTS = {
    "no_max_subtraction": ("s += std::exp(logit(x, i * N + j, dtype) - m);", "s += std::exp(logit(x, i * N + j, dtype));"),
    "base_two_exponential": ("s += std::exp(logit(", "s += std::exp2(logit("),
    "log_base_two": ("static_cast<float>(std::log(s) -", "static_cast<float>(std::log2(s) -"),
    "first_term_missing": ("    for (int64_t j = 0; j < N; ++j) s +=", "    for (int64_t j = (N > 1 ? 1 : 0); j < N; ++j) s +="),
    "mean_instead_of_sum": ("static_cast<float>(std::log(s) -", "static_cast<float>(std::log(s / (double)N) -"),
    "sign_of_the_picked_logit": ("- (logit(x, i * N + t, dtype) - m));", "+ (logit(x, i * N + t, dtype) - m));"),
    "target_of_the_wrong_row": ("- (logit(x, i * N + t, dtype) - m));", "- (logit(x, ((i + 1) % (r1 > 1 ? r1 : 1)) * N + t, dtype) - m));"),
    "target_off_by_one": ("- (logit(x, i * N + t, dtype) - m));", "- (logit(x, i * N + (t + 1) % N, dtype) - m));"),
    "max_not_added_back_to_lse_but_loss_uses_lse": ("static_cast<float>(std::log(s) - (logit(x, i * N + t, dtype) - m));",
                                                    "static_cast<float>(std::log(s) - logit(x, i * N + t, dtype));"),
    "ignored_rows_not_zero": ("      loss[i] = 0.0f;                         // ignored row", "      loss[i] = static_cast<float>(lse);"),
    "ignore_only_negative": ("if (t < 0 || t >= N) {", "if (t < 0) { loss[i] = 0.0f; } else if (t >= N) { loss[i] = 1.0f; } else if (false) {"),
    "rounds_through_bf16_width": ("static_cast<float>(std::log(s) - (logit(x, i * N + t, dtype) - m));",
                                  "static_cast<float>(std::ldexp(std::nearbyint(std::ldexp(std::log(s) - (logit(x, i * N + t, dtype) - m), 20)), -20));"),
    "half_decoded_with_wrong_bias": ("v = std::ldexp(static_cast<double>(frac + 1024), ex - 25);", "v = std::ldexp(static_cast<double>(frac + 1024), ex - 24);"),
    "bf16_shift": ("static_cast<uint32_t>(h) << 16;", "static_cast<uint32_t>(h) << 15;"),
}


ROWSUM_SRC = os.path.join(ROOT, "oracle", "rowsum_oracle.cpp")
ROWSUM_PINS = os.path.join(ROOT, "tests", "test_rowsum_oracle_pins.py")

ROWSUM_MUTANTS = {
    "first_term_missing": ("    for (int64_t j = 0; j < N; ++j) {\n      const double v", "    for (int64_t j = (N > 1 ? 1 : 0); j < N; ++j) {\n      const double v"),
    "last_term_missing": ("    for (int64_t j = 0; j < N; ++j) {\n      const double v", "    for (int64_t j = 0; j + 1 < N || j == 0; ++j) {\n      const double v"),
    "mean_instead_of_sum": ("y[i] = static_cast<float>(total);", "y[i] = static_cast<float>(total / (double)N);"),
    "fp32_running_total": ("double total = 0.0, total_abs = 0.0;", "float total = 0.0f; double total_abs = 0.0;"),
    "sum_of_magnitudes_as_result": ("      total += v;\n", "      total += std::fabs(v);\n"),
    "signed_sum_as_magnitudes": ("total_abs += std::fabs(v);", "total_abs += v;"),
    "column_major_read": ("const double v = element(x, i * N + j, dtype);", "const double v = element(x, (i + j * (end - first)) % ((end - first) * N) + first * N, dtype);"),
    "next_rows_element": ("const double v = element(x, i * N + j, dtype);", "const double v = element(x, i * N + (j + 1 < N ? j + 1 : j), dtype);"),
    "result_rounded_to_bf16_width": ("y[i] = static_cast<float>(total);", "y[i] = static_cast<float>(std::ldexp(std::nearbyint(std::ldexp(total, 7 - std::ilogb(total == 0 ? 1.0 : total))), std::ilogb(total == 0 ? 1.0 : total) - 7));"),
    "result_truncated": ("y[i] = static_cast<float>(total);", "{ float r = static_cast<float>(total); if (std::fabs((double)r) > std::fabs(total)) r = std::nextafterf(r, 0.0f); y[i] = r; }"),
    "half_decoded_with_wrong_bias": ("magnitude = std::ldexp(static_cast<double>(1024 + fraction), exponent - 25);", "magnitude = std::ldexp(static_cast<double>(1024 + fraction), exponent - 24);"),
    "half_subnormals_flushed": ("else if (exponent == 0) magnitude = std::ldexp(static_cast<double>(fraction), -24);", "else if (exponent == 0) magnitude = 0.0;"),
    "half_hidden_bit_missing": ("static_cast<double>(1024 + fraction), exponent - 25", "static_cast<double>(fraction), exponent - 25"),
    "bf16_shift": ("static_cast<uint32_t>(bits) << 16;", "static_cast<uint32_t>(bits) << 15;"),
    "sign_lost": ("return negative ? -magnitude : magnitude;", "return magnitude;"),
    "half_nan_read_as_infinity": ("magnitude = fraction != 0 ? std::nan(\"\") : INFINITY;", "magnitude = INFINITY;"),
}


def _build(source_text: str, out_dir, name: str) -> str:
    cpp = os.path.join(out_dir, f"{name}.cpp")
    so = os.path.join(out_dir, f"{name}.so")
    with open(cpp, "w") as f:
        f.write(source_text)
    subprocess.run(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-pthread", "-o", so, cpp],
                   check=True)
    return so


def _run_pins(lib_path: str, var: str = "RMSNORM_ORACLE_LIB", pins: str = PINS) -> int:
    env = dict(os.environ)
    env[var] = lib_path
    proc = subprocess.run([sys.executable, "-m", "pytest", pins, "-x", "-q", "-p", "no:cacheprovider"],
                          cwd=ROOT, env=env, capture_output=True, text=True)
    return proc.returncode


def test_unmodified_oracle_passes_its_pins_through_the_same_route(tmp_path):
    so = _build(open(SRC).read(), str(tmp_path), "pristine")
    assert _run_pins(so) == 0


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(tmp_path, name):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found; update the test"
    so = _build(text.replace(old, new), str(tmp_path), name)
    assert _run_pins(so) != 0, f"no pin noticed the planted mistake '{name}'"


def test_unmodified_softmax_oracle_passes_its_pins_through_the_same_route(tmp_path):
    so = _build(open(SOFTMAX_SRC).read(), str(tmp_path), "pristine_softmax")
    assert _run_pins(so, "SOFTMAX_ORACLE_LIB", SOFTMAX_PINS) == 0


@pytest.mark.parametrize("name", sorted(SOFTMAX_MUTANTS))
def test_planted_softmax_mistake_is_caught(tmp_path, name):
    old, new = SOFTMAX_MUTANTS[name]
    text = open(SOFTMAX_SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found; update the test"
    so = _build(text.replace(old, new), str(tmp_path), name)
    assert _run_pins(so, "SOFTMAX_ORACLE_LIB", SOFTMAX_PINS) != 0, \
        f"no pin noticed the planted mistake '{name}'"


def test_unmodified_layernorm_oracle_passes_its_pins_through_the_same_route(tmp_path):
    so = _build(open(LAYERNORM_SRC).read(), str(tmp_path), "pristine_layernorm")
    assert _run_pins(so, "LAYERNORM_ORACLE_LIB", LAYERNORM_PINS) == 0


@pytest.mark.parametrize("name", sorted(LAYERNORM_MUTANTS))
def test_planted_layernorm_mistake_is_caught(tmp_path, name):
    old, new = LAYERNORM_MUTANTS[name]
    text = open(LAYERNORM_SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found; update the test"
    so = _build(text.replace(old, new), str(tmp_path), name)
    assert _run_pins(so, "LAYERNORM_ORACLE_LIB", LAYERNORM_PINS) != 0, \
        f"no pin noticed the planted mistake '{name}'"


def test_unmodified_crossentropy_oracle_passes_its_pins_through_the_same_route(tmp_path):
    so = _build(open(CE_SRC).read(), str(tmp_path), "pristine_ce")
    assert _run_pins(so, "CROSSENTROPY_ORACLE_LIB", CE_PINS) == 0


@pytest.mark.parametrize("name", sorted(CE_MUTANTS))
def test_planted_crossentropy_mistake_is_caught(tmp_path, name):
    old, new = CE_MUTANTS[name]
    text = open(CE_SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found; update the test"
    so = _build(text.replace(old, new), str(tmp_path), name)
    assert _run_pins(so, "CROSSENTROPY_ORACLE_LIB", CE_PINS) != 0, \
        f"no pin noticed the planted mistake '{name}'"


def test_unmodified_rowsum_oracle_passes_its_pins_through_the_same_route(tmp_path):
    so = _build(open(ROWSUM_SRC).read(), str(tmp_path), "pristine_rowsum")
    assert _run_pins(so, "ROWSUM_ORACLE_LIB", ROWSUM_PINS) == 0


@pytest.mark.parametrize("name", sorted(ROWSUM_MUTANTS))
def test_planted_rowsum_mistake_is_caught(tmp_path, name):
    old, new = ROWSUM_MUTANTS[name]
    text = open(ROWSUM_SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found; update the test"
    so = _build(text.replace(old, new), str(tmp_path), name)
    assert _run_pins(so, "ROWSUM_ORACLE_LIB", ROWSUM_PINS) != 0, \
        f"no pin noticed the planted mistake '{name}'"
