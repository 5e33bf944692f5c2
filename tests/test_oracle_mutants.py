"""Do the pins bite?  Each case plants one plausible mistake (a dropped term, a wrong sign, index or constant,
a swapped operand) in a copy of oracle/gg_oracle.c, builds it, lets the oracle's Python front-end call that
build, and runs one pin of the other test files: the pin has to fail.  Everything happens on the CPU.

What is not covered here on purpose: the conventions of the sampler's random stream (which Philox word feeds
which draw, cosine or sine in Box-Muller, 23 or 24 bits per uniform).  They are this build's choice, any
of them samples the same distribution, and nothing outside the oracle fixes them."""
import concurrent.futures
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC_DIR = os.path.join(os.path.dirname(HERE), "oracle")

RHO = "return 2.0 * lgamma(2.0 / b) - lgamma(1.0 / b) - lgamma(3.0 / b);"
ALPHA = "return sqrt(m2 * exp(lgamma(1.0 / beta) - lgamma(3.0 / beta)));"
INIT = "return sqrt(xi / (double)d_in * exp(lgamma(1.0 / shape) - lgamma(3.0 / shape)));"
EGLEN = "return 2u * fl - (uint32_t)k + 1u;"
PEN = "p = lam * b * pow(fabs(v) / a, b - 1.0) * s / a;"
GCT_COEF = "double coef = 4.0 * (double)inv_delta / ((double)n_rate * ln2);"
RG_COEF = "double coef = (double)scale * 4.0 * (double)inv_delta / ((double)n_rate * ln2);"
FUSED_PEN = "orc_penalty_grad(xs, dtype, n, a32, b32, lambda, grad + lo, accumulate);"

# (name, text in the oracle, replacement, test module, test function, its arguments)
MUTANTS = [
    ("rho: Gamma(2/b) not squared", RHO, RHO.replace("2.0 * lgamma(2.0", "1.0 * lgamma(2.0"),
     "test_oracle_stats", "test_rho_closed_forms", ()),
    ("rho: Gamma(2/b) and Gamma(3/b) swapped", RHO, "return 2.0 * lgamma(3.0 / b) - lgamma(1.0 / b) - lgamma(2.0 / b);",
     "test_oracle_stats", "test_rho_matches_integrated_density", (0.8,)),
    ("Eq. 2: Gamma ratio inverted", ALPHA, "return sqrt(m2 * exp(lgamma(3.0 / beta) - lgamma(1.0 / beta)));",
     "test_oracle_stats", "test_fit_from_exact_moments", (1.0, 1.0, 2.0)),
    ("Eq. 2: square root dropped", ALPHA, "return (m2 * exp(lgamma(1.0 / beta) - lgamma(3.0 / beta)));",
     "test_oracle_stats", "test_fit_from_exact_moments", (1.0, 1.0, 2.0)),
    ("Eq. 5: activation factor dropped", INIT, INIT.replace("sqrt(xi /", "sqrt(1.0 /"),
     "test_oracle_stats", "test_init_alpha_reduces_to_he_at_shape_2", (11008, 2.0)),
    ("Eq. 5: Gamma ratio inverted", INIT, "return sqrt(xi / (double)d_in * exp(lgamma(3.0 / shape) - lgamma(1.0 / shape)));",
     "test_oracle_stats", "test_init_alpha_gives_variance_xi_over_din", (0.5,)),
    ("moments: |x| without the absolute value", "s1 += (double)fabsf(v);", "s1 += (double)v;",
     "test_oracle_stats", "test_moments_small_by_hand", ()),
    ("moment ratio: first moment not squared", "double rho = m1 * m1 / m2;", "double rho = m1 / m2;",
     "test_oracle_stats", "test_fit_from_exact_moments", (2.0, 0.5641895835477563, 0.5)),
    ("bisection moves the wrong end", "if (log_rho(mid) < target)", "if (log_rho(mid) > target)",
     "test_oracle_stats", "test_solve_inverts_integrated_rho", (0.8,)),
    ("degenerate unit reports shape 1", "out->flags = ORC_DEGENERATE;\n        out->beta = 2.0;",
     "out->flags = ORC_DEGENERATE;\n        out->beta = 1.0;", "test_oracle_stats", "test_fit_degenerate_empty_nonfinite", ()),
    ("compression ratio inverted", "return 1.0 - mean_bits / fl_bits;", "return 1.0 - fl_bits / mean_bits;",
     "test_oracle_stats", "test_compression_ratio_matches_paper_tables", ()),
    ("quantiser rounds up", "rintf(t) : floorf(t);", "rintf(t) : ceilf(t);",
     "test_oracle_rate", "test_quantize_power_of_two_step_is_exact_floor", ()),
    ("quantiser truncates toward zero", "rintf(t) : floorf(t);", "rintf(t) : truncf(t);",
     "test_oracle_rate", "test_quantize_dead_zone_is_asymmetric_under_floor", ()),
    ("quantiser clamps at 2^31", "const float lim = 1073741824.0f; /* 2^30 */", "const float lim = 2147483648.0f;",
     "test_oracle_rate", "test_quantize_nan_inf_and_clamp", ()),
    ("NaN quantises to 1", "*flags |= ORC_NONFINITE;\n        return 0;", "*flags |= ORC_NONFINITE;\n        return 1;",
     "test_oracle_rate", "test_quantize_nan_inf_and_clamp", ()),
    ("saturation flag one symbol late", "if (umax >= 2147483647u) flags |= ORC_SATURATED;",
     "if (umax > 2147483647u) flags |= ORC_SATURATED;", "test_oracle_rate", "test_quantize_nan_inf_and_clamp", ()),
    ("Map: odd and even sides swapped", "if (q < 0) return (uint32_t)(-2 * (int64_t)q);",
     "if (q < 0) return (uint32_t)(-2 * (int64_t)q - 1);", "test_oracle_rate", "test_map_paper_table", ()),
    ("Map: 2q+1 for positives", "return (uint32_t)(2 * (int64_t)q - 1);", "return (uint32_t)(2 * (int64_t)q + 1);",
     "test_oracle_rate", "test_map_bijection_parity_and_order", ()),
    ("EG length: the +1 dropped", EGLEN, "return 2u * fl - (uint32_t)k;", "test_oracle_rate", "test_eg_len_hand_values", ()),
    ("EG length: +k instead of -k", EGLEN, "return 2u * fl + (uint32_t)k + 1u;",
     "test_oracle_rate", "test_eg_len_equals_codeword_length", (3,)),
    ("EG length: 2^k not added to the symbol", "uint64_t v = (uint64_t)u + ((uint64_t)1 << k);\n    uint32_t fl = 0;",
     "uint64_t v = (uint64_t)u + 1;\n    uint32_t fl = 0;", "test_oracle_rate", "test_eg_code_is_prefix_free_kraft", ()),
    ("histogram: last regular bin counted as clamped", "if (u > (uint32_t)(nbins - 1)) {", "if (u >= (uint32_t)(nbins - 1)) {",
     "test_oracle_rate", "test_rate_matches_brute_force", (0.6, 8, 0, 64)),
    ("entropy in nats", "H -= p * log2(p);", "H -= p * log(p);",
     "test_oracle_rate", "test_laplace_closed_form_entropy_and_eg_rate", ()),
    ("entropy: probabilities over n+1", "double p = (double)hist[b] / (double)n;", "double p = (double)hist[b] / (double)(n + 1);",
     "test_oracle_rate", "test_rate_matches_brute_force", (2.0, 4, 2, 32)),
    ("fixed-length bits of an all-zero unit are 0", "out->fl_bits = bit_length(umax) > 1u ? bit_length(umax) : 1u;",
     "out->fl_bits = bit_length(umax);", "test_oracle_rate", "test_rate_hand_cases", ()),
    ("bucket: step = alpha times the divisor", "a32 / delta_div : delta[s];", "a32 * delta_div : delta[s];",
     "test_oracle_rate", "test_fused_segmented_equals_per_segment_calls", (False,)),
    ("bucket: bf16 units addressed with 4-byte strides", "(size_t)lo * esz;", "(size_t)lo * 4;",
     "test_oracle_rate", "test_fused_segmented_equals_per_segment_calls", (True,)),
    ("bucket: alpha and beta swapped in the penalty", FUSED_PEN, FUSED_PEN.replace("a32, b32", "b32, a32"),
     "test_oracle_rate", "test_fused_segmented_equals_per_segment_calls", (False,)),
    ("bucket: every unit's penalty written at the start", FUSED_PEN, FUSED_PEN.replace("grad + lo", "grad"),
     "test_oracle_rate", "test_fused_segmented_equals_per_segment_calls", (False,)),
    ("penalty: exponent beta instead of beta-1", PEN, PEN.replace("b - 1.0", "b"),
     "test_oracle_penalty_sampler", "test_penalty_is_derivative_of_prior_exponent", (1.3,)),
    ("penalty: the final 1/alpha dropped", PEN, PEN.replace("* s / a;", "* s;"),
     "test_oracle_penalty_sampler", "test_penalty_laplace_and_gaussian_closed_forms", ()),
    ("penalty: factor beta dropped", PEN, PEN.replace("lam * b *", "lam *"),
     "test_oracle_penalty_sampler", "test_penalty_laplace_and_gaussian_closed_forms", ()),
    ("penalty: sign flipped", "double s = v > 0.0 ? 1.0 : -1.0;\n            p = lam", "double s = v > 0.0 ? -1.0 : 1.0;\n            p = lam",
     "test_oracle_penalty_sampler", "test_penalty_laplace_and_gaussian_closed_forms", ()),
    ("bf16 input read from the wrong half", "((const uint16_t *)x)[i] << 16;", "((const uint16_t *)x)[i] << 15;",
     "test_oracle_penalty_sampler", "test_penalty_zero_odd_symmetry_accumulate_bf16", ()),
    ("bf16 rounding: ties away from zero", "bits += 0x7fffu + lsb;", "bits += 0x8000u;",
     "test_oracle_penalty_sampler", "test_bf16_rounding_is_nearest_even", ()),
    ("bf16 rounding: truncation", "bits += 0x7fffu + lsb;", "bits += 0u;",
     "test_oracle_penalty_sampler", "test_bf16_rounding_is_nearest_even", ()),
    ("Philox: multipliers swapped", "const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;",
     "const uint64_t M0 = 0xCD9E8D57u, M1 = 0xD2511F53u;", "test_oracle_penalty_sampler", "test_philox_known_answers", ()),
    ("Philox: nine rounds", "for (int r = 0; r < 10; ++r) {", "for (int r = 0; r < 9; ++r) {",
     "test_oracle_penalty_sampler", "test_philox_known_answers", ()),
    ("Philox: key increments swapped", "k0 += W0;\n        k1 += W1;", "k0 += W1;\n        k1 += W0;",
     "test_oracle_penalty_sampler", "test_philox_known_answers", ()),
    ("Gamma draw: d = a - 1/2", "- 1.0 / 3.0;\n    *c", "- 1.0 / 2.0;\n    *c",
     "test_oracle_penalty_sampler", "test_sampler_laplace_case_is_exponential", ()),
    ("Gamma draw: c = 1/sqrt(3d), a valid but loose envelope", "*c = 1.0 / sqrt(9.0 * *d);", "*c = 1.0 / sqrt(3.0 * *d);",
     "test_oracle_penalty_sampler", "test_sampler_rejection_step_has_the_published_efficiency", (1.0,)),
    ("Gamma draw: envelope too narrow", "*c = 1.0 / sqrt(9.0 * *d);", "*c = 1.0 / sqrt(12.0 * *d);",
     "test_oracle_penalty_sampler", "test_sampler_laplace_case_is_exponential", ()),
    ("Gamma draw: acceptance test with d - dv negated", "if (lu < 0.5 * z * z + d - d * v + d * log(v)) {",
     "if (lu < 0.5 * z * z - d + d * v + d * log(v)) {", "test_oracle_penalty_sampler", "test_sampler_laplace_case_is_exponential", ()),
    ("Gamma draw: square instead of cube", "double v = t * t * t;", "double v = t * t;",
     "test_oracle_penalty_sampler", "test_sampler_laplace_case_is_exponential", ()),
    ("normal draw: variance halved", "sqrt(-2.0 * log(unit_open(w[0])))", "sqrt(-1.0 * log(unit_open(w[0])))",
     "test_oracle_penalty_sampler", "test_sampler_laplace_case_is_exponential", ()),
    ("sampler: shape < 1 not boosted down", "if (boost) mag *= unit_open(w3_first);", "",
     "test_oracle_penalty_sampler", "test_sampler_general_shape_transforms_to_gamma", (1.5,)),
    ("sampler: G^beta instead of G^(1/beta)", "double mag = pow(gam, a);", "double mag = pow(gam, (double)beta);",
     "test_oracle_penalty_sampler", "test_sampler_general_shape_transforms_to_gamma", (0.5,)),
    ("sampler: no sign", "if (w3_first & 1u) xval = -xval;", "",
     "test_oracle_penalty_sampler", "test_sampler_general_shape_transforms_to_gamma", (0.8,)),
    ("GCT: curvature with 1 + g/ghat", "(1.0 - gi / (", "(1.0 + gi / (", "test_oracle_next", "test_gct_step_by_hand", ()),
    ("GCT: curvature without 1/eta", "h = (1.0 / (double)eta) * (1.0 - gi", "h = (1.0) * (1.0 - gi",
     "test_oracle_next", "test_gct_step_by_hand", ()),
    ("GCT: eps dropped from the denominator", "((double)g_hat_prev[i] + (double)eps)", "((double)g_hat_prev[i])",
     "test_oracle_next", "test_gct_eps_guards_a_vanished_previous_gradient", ()),
    ("GCT: rate slope halved", GCT_COEF, GCT_COEF.replace("4.0 *", "2.0 *"), "test_oracle_next", "test_gct_step_by_hand", ()),
    ("GCT: weight moves up the gradient", "(double)w[i] - (double)eta * (double)ghat32", "(double)w[i] + (double)eta * (double)ghat32",
     "test_oracle_next", "test_gct_first_step_is_plain_sgd", ()),
    ("GCT: rate term subtracted", "double ghat = gi + (double)lambda * dR * h;", "double ghat = gi - (double)lambda * dR * h;",
     "test_oracle_next", "test_gct_step_by_hand", ()),
    ("GCT: the first step uses the curvature too", "if (!first_step)\n            h =", "if (1)\n            h =",
     "test_oracle_next", "test_gct_first_step_is_plain_sgd", ()),
    ("rate gradient: factor 2 lost", RG_COEF, RG_COEF.replace("4.0 *", "2.0 *"),
     "test_oracle_next", "test_rate_grad_is_slope_of_smoothed_mean_eg_length", ()),
    ("rate gradient: ln 2 lost", RG_COEF, RG_COEF.replace("((double)n_rate * ln2)", "((double)n_rate)"),
     "test_oracle_next", "test_rate_grad_is_slope_of_smoothed_mean_eg_length", ()),
    ("rate gradient: 2^k replaced by 1", "float d = (float)(coef * s / ((double)u + (double)((uint64_t)1 << eg_k)));",
     "float d = (float)(coef * s / ((double)u + 1.0));", "test_oracle_next",
     "test_rate_grad_sign_zero_scale_accumulate_and_gct_consistency", ()),
    ("EG stream: one zero too many in the prefix", "pos += (uint64_t)(L - 1 - eg_k); /* zero prefix */", "pos += (uint64_t)(L - eg_k);",
     "test_oracle_next", "test_eg_stream_known_bits", ()),
    ("EG stream: bits filled from the low end of a byte", "(uint8_t)(0x80u >> (pos & 7u));", "(uint8_t)(0x01u << (pos & 7u));",
     "test_oracle_next", "test_eg_stream_known_bits", ()),
    ("EG decoder: code one bit short", "int L = zeros + eg_k + 1;", "int L = zeros + eg_k;",
     "test_oracle_next", "test_eg_stream_round_trip_and_length", (1,)),
    ("EG decoder: subtracts 1 instead of 2^k", "u[cnt++] = (uint32_t)(v - ((uint64_t)1 << eg_k));", "u[cnt++] = (uint32_t)(v - 1);",
     "test_oracle_next", "test_eg_stream_round_trip_and_length", (3,)),
    ("reconstruction at the middle of the cell", "volatile float v = (float)q[i] * delta;", "volatile float v = ((float)q[i] + 0.5f) * delta;",
     "test_oracle_next", "test_dequantize_gives_the_lower_end_of_the_quantiser_cell", ()),
    ("reconstruction: accumulate overwrites", "volatile float sum = out[i] + v;\n            out[i] = sum;", "out[i] = v;",
     "test_oracle_next", "test_dequantize_gives_the_lower_end_of_the_quantiser_cell", ()),
    ("Huffman: a single symbol costs 0 bits", "if (m == 1) return 1.0;", "if (m == 1) return 0.0;",
     "test_oracle_next", "test_huffman_textbook_and_bounds", ()),
    ("Huffman: merges the larger of the two queues' heads", "leaf[li] <= node[ni]))", "leaf[li] > node[ni]))",
     "test_oracle_next", "test_huffman_textbook_and_bounds", ()),
]


RUN_PIN = """
import importlib, sys, traceback
sys.path[:0] = [{root!r}, {tests!r}]
import oracle
pin = getattr(importlib.import_module({module!r}), {function!r})
try:
    pin(*{args!r})                      # the pin holds for the oracle as it is
except BaseException:
    traceback.print_exc()
    sys.exit(3)
oracle._lib = oracle.load({so!r})
pin(*{args!r})                          # and has to fail for the altered build (uncaught: exit status 1)
"""


def _run(case, source, header, folder):
    name, old, new, module, function, args = case
    if source.count(old) != 1:
        return "the oracle's text changed: bring this case up to date"
    os.makedirs(folder)
    with open(os.path.join(folder, "gg_oracle.c"), "w") as f:
        f.write(source.replace(old, new))
    with open(os.path.join(folder, "gg_oracle.h"), "w") as f:
        f.write(header)
    so = os.path.join(folder, "libgg_oracle_altered.so")
    subprocess.run(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off", "-o", so,
                    os.path.join(folder, "gg_oracle.c"), "-lm"], check=True)
    script = RUN_PIN.format(root=os.path.dirname(HERE), tests=HERE, so=so, module=module, function=function, args=args)
    # A process of its own, under a time limit: a mistake may also make the oracle loop or crash, and either
    # counts as noticed.
    try:
        done = subprocess.run([sys.executable, "-c", script], capture_output=True, text=True, timeout=30)
    except subprocess.TimeoutExpired:
        return None
    if done.returncode == 0:
        return "the pin passed on the altered oracle"
    if done.returncode == 3:
        return "the pin fails on the oracle as it is:\n" + done.stderr[-2000:]
    return None


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    """Every case built and run once, eight at a time: name -> None (noticed) or what went wrong."""
    with open(os.path.join(SRC_DIR, "gg_oracle.c")) as f:
        source = f.read()
    with open(os.path.join(SRC_DIR, "gg_oracle.h")) as f:
        header = f.read()
    base = str(tmp_path_factory.mktemp("altered"))
    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as pool:
        jobs = [pool.submit(_run, case, source, header, os.path.join(base, str(i))) for i, case in enumerate(MUTANTS)]
        return {case[0]: job.result() for case, job in zip(MUTANTS, jobs)}


@pytest.mark.parametrize("name", [m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_its_pin(name, outcomes):
    assert outcomes[name] is None, outcomes[name]
