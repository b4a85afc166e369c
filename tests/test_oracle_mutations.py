"""The pins must be able to fail: each case plants one plausible mistake in a COPY of the oracle's
source (never in the GPU library), builds it, and runs the pin suite against it in a subprocess;
the suite has to report a failure.  CPU only."""
import os
import subprocess
import sys

import pytest

from conftest import ROOT

SOURCE = os.path.join(ROOT, "oracle", "fbsr_oracle.cpp")

# name -> the pins (pytest -k expression) that are expected to notice it; running only those keeps the
# suite quick.  The planted mistake must make at least one of them fail.
WATCHERS = {'srf_half_term_dropped': 'exhaustive_round_up_counts and 2-0', 'srff_strict_compare': 'representables_are_fixed or exhaustive_round_up_counts and 2-0', 'rne_ties_to_odd': 'rne_matches_library_cast', 'src_inner_round_is_floor': 'src_ties or closed_form_bias_fp32_to_bf16', 'src_ties_away': 'src_ties', 'subnormal_clamp_dropped': 'rne_matches_library_cast', 'philox_multipliers_swapped': 'philox_known', 'philox_nine_rounds': 'philox_known', 'slot_uses_n_not_w': 'random_bits_are_slices', 'overflow_tie_goes_down': 'specials_and_out_of_range', 'e4m3_overflows_to_nan': 'specials_and_out_of_range', 'sign_lost': 'rne_matches_library_cast', 'exponent_carry_missing': 'rne_matches_library_cast', 'sgd_two_roundings': 'sgd_is_one_fma', 'sgd_step_not_in_key': 'sgd_is_one_fma', 'stats_error_sign': 'stats_sum_is_the_exact', 'stats_ulp_of_wrong_format': 'stats_sum_is_the_exact', 'qat_bias_correction_dropped': 'qat_step_tracks', 'qat_weight_decay_sign': 'qat_step_tracks', 'qat_sum_not_rounded_to_16_bits': 'qat_step_structure', 'widen_fp16_bias': 'widening_matches',
            'tno_is_tne': 'deterministic_modes', 'ta_is_strict': 'deterministic_modes',
            'src_odd_parity': 'ties_to_odd', 'generic_overflow_tie_parity': 'overflow_and_specials',
            'generic_negative_zero_kept': 'overflow_and_specials', 'generic_subnormal_scale': 'published_value_sets',
            'generic_nan_sign_dropped': 'overflow_and_specials',
            'qat8_step_not_in_key': 'qat_step_structure_in_binary8p4', 'qat8_nan_becomes_max': 'qat_step_structure_in_binary8p4',
            'qat_eps_inside_the_root': 'eps_outside_the_root', 'stats_ulp_not_clamped_for_subnormals': 'exact_rational_sums',
            'stats8_ulp_ignores_the_descriptors_bias': 'stats_under_an_ocp_descriptor or test_oracle_format8 and exact_rational_sums',
            'stats8_first_bin_ignored': 'stats_under_an_ocp_descriptor', 'stats8_sum_y_takes_the_input': 'test_oracle_format8 and exact_rational_sums', 'stats8_error_sign': 'test_oracle_format8 and exact_rational_sums',
            'stats_sum_y_takes_the_input': 'exact_rational_sums'}

MUTATIONS = [
    ("srf_half_term_dropped", "std::ldexp((double)(2 * n + 1), -(N + 1))", "std::ldexp((double)(2 * n), -(N + 1))"),
    ("srff_strict_compare", "return delta >= 1.0 - std::ldexp((double)n, -N);", "return delta > 1.0 - std::ldexp((double)n, -N);"),
    ("rne_ties_to_odd", "std::fmod(fl, 2.0) == 1.0", "std::fmod(fl, 2.0) == 0.0"),
    ("src_inner_round_is_floor", "std::nearbyint(std::ldexp(delta, N))", "std::floor(std::ldexp(delta, N))"),
    ("src_ties_away", "std::nearbyint(std::ldexp(delta, N))", "std::floor(std::ldexp(delta, N) + 0.5)"),
    ("subnormal_clamp_dropped", "return lg > 1 - f.B ? lg : 1 - f.B;", "return lg;"),
    ("philox_multipliers_swapped", "M0 = 0xD2511F53ull, M1 = 0xCD9E8D57ull", "M0 = 0xCD9E8D57ull, M1 = 0xD2511F53ull"),
    ("philox_nine_rounds", "round < 10", "round < 9"),
    ("slot_uses_n_not_w", "const unsigned bit = slot * (unsigned)W;", "const unsigned bit = slot * (unsigned)N;"),
    ("overflow_tie_goes_down", "a < f.M + half_ulp_M ? m_code", "a <= f.M + half_ulp_M ? m_code"),
    ("e4m3_overflows_to_nan", "if (!f.has_inf) return sign_code | m_code;", "if (!f.has_inf) return sign_code | f.nan_code;"),
    ("sign_lost", "return sign_code | encode_magnitude(sigma, et, f);", "return encode_magnitude(sigma, et, f);"),
    ("exponent_carry_missing", "    sigma = (int64_t)1 << (f.P - 1);\n    et += 1;", "    sigma = (int64_t)1 << (f.P - 1);"),
    ("sgd_two_roundings", "std::fmaf(-lr, g[j], bf16_to_float(w[j]))", "(-lr * g[j] + bf16_to_float(w[j]))"),
    ("sgd_step_not_in_key", "random_bits(seed, step, offset + j, nbits);\n    w[j]", "random_bits(seed, 0, offset + j, nbits);\n    w[j]"),
    ("stats_error_sign", "const double e = (y - (double)x[j]) / oracle_ulp(x[j], fmt);", "const double e = ((double)x[j] - y) / oracle_ulp(x[j], fmt);"),
    ("stats_ulp_of_wrong_format", "return std::ldexp(1.0, rounding_exponent(a, f) - f.P + 1);", "return std::ldexp(1.0, rounding_exponent(a, f) - f.P);"),
    ("qat_bias_correction_dropped", "bf16_to_float(mq) / a.bias_corr1", "bf16_to_float(mq)"),
    ("qat_weight_decay_sign", "std::fmaf(a.weight_decay, w, ratio)", "std::fmaf(-a.weight_decay, w, ratio)"),
    ("qat_sum_not_rounded_to_16_bits", "bf16_to_float(to_bf16_rne(w + u16));", "(w + u16);"),
    ("widen_fp16_bias", "Format{16, 11, 15, 65504.0", "Format{16, 11, 16, 65504.0"),
    ("tno_is_tne", "delta == 0.5 && std::fmod(fl, 2.0) == 0.0", "delta == 0.5 && std::fmod(fl, 2.0) == 1.0"),
    ("ta_is_strict", "return delta >= 0.5;", "return delta > 0.5;"),
    ("src_odd_parity", "r == 0.5 && std::fmod(lo, 2.0) == 0.0", "r == 0.5 && std::fmod(lo, 2.0) == 1.0"),
    ("generic_overflow_tie_parity", "std::fmod(f.M / ulp_M, 2.0) == 1.0", "std::fmod(f.M / ulp_M, 2.0) == 0.0"),
    ("generic_negative_zero_kept", "if (mag == 0 && !g.neg_zero) return 0u;", ""),
    ("generic_subnormal_scale", "std::ldexp(1.0, 1 - f.B);      // Eq. (1)", "std::ldexp(1.0, -f.B);      // Eq. (1)"),
    ("qat8_step_not_in_key", "random_bits(seed, step, offset + j, nbits) : 0;\n      code = round_one8", "random_bits(seed, 0, offset + j, nbits) : 0;\n      code = round_one8"),
    ("qat8_nan_becomes_max", "code = g.nan_code >= 0 ? (uint32_t)g.nan_code : (uint32_t)g.max_code;", "code = (uint32_t)g.max_code;"),
    ("generic_nan_sign_dropped", "(uint32_t)g.nan_code | (g.nan_signed ? sign_code : 0u)", "(uint32_t)g.nan_code"),
    ("qat_eps_inside_the_root", "mh / (std::sqrt(vh) + a.eps)", "mh / std::sqrt(vh + a.eps)"),
    ("stats_ulp_not_clamped_for_subnormals", "return std::ldexp(1.0, rounding_exponent(a, f) - f.P + 1);",
     "return std::ldexp(1.0, std::ilogb(a) - f.P + 1);"),
    ("stats_sum_y_takes_the_input", "oracle_ulp(x[j], fmt);\n    double* s = stats + 4 * bin;\n    s[0] += 1.0;\n    s[1] += y;",
     "oracle_ulp(x[j], fmt);\n    double* s = stats + 4 * bin;\n    s[0] += 1.0;\n    s[1] += (double)x[j];"),
    ("stats8_sum_y_takes_the_input", "/ ulp;\n    double* s = stats + 4 * bin;\n    s[0] += 1.0;\n    s[1] += y;",
     "/ ulp;\n    double* s = stats + 4 * bin;\n    s[0] += 1.0;\n    s[1] += (double)x[j];"),
    ("stats8_ulp_ignores_the_descriptors_bias", "std::ldexp(1.0, rounding_exponent(a, g.f) - g.f.P + 1) : 1.0;",
     "std::ldexp(1.0, std::ilogb(a == 0.0 ? 1.0 : a) - g.f.P + 1) : 1.0;"),
    ("stats8_first_bin_ignored", "const uint64_t bin = i / group - first_bin;\n    const uint64_t r = variant_draws(variant)",
     "const uint64_t bin = i / group;\n    const uint64_t r = variant_draws(variant)"),
    ("stats8_error_sign", "const double e = (y - (double)x[j]) / ulp;", "const double e = ((double)x[j] - y) / ulp;"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_is_caught(tmp_path, name, old, new):
    text = open(SOURCE).read()
    assert text.count(old) == 1, "mutation target not found exactly once: %s" % name
    src = tmp_path / "mutant.cpp"
    lib = tmp_path / "libmutant.so"
    src.write_text(text.replace(old, new))
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared", "-pthread",
                           "-o", str(lib), str(src)])
    env = dict(os.environ, FBSR_ORACLE_LIB=str(lib))
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                          os.path.join(ROOT, "tests", "test_oracle_format8.py"), "-x", "-q",
                          "-p", "no:cacheprovider", "-k", WATCHERS[name]], env=env, cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    assert run.returncode != 0, "no pin noticed the planted mistake '%s'" % name
    assert b"failed" in run.stdout or b"error" in run.stdout.lower()
