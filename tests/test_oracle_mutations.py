"""Are the pins strong enough?  Each case plants one plausible mistake in a COPY of the oracle's C
source (a dropped factor, a wrong sign or index, a strictness flip), builds it, and checks that at
least one of the oracle's pins fails on it.  CPU only; the real oracle is restored afterwards."""
import ctypes as C
import os
import subprocess

import pytest

import oracle
import test_oracle_cett as t_cett
import test_oracle_ffn as t_ffn
import test_oracle_geglu as t_geglu
import test_oracle_relu as t_relu
import test_oracle_signals as t_sig
import test_oracle_static_mask as t_mask

SRC = os.path.join(os.path.dirname(oracle.__file__), "clada_oracle.c")

FFN_PINS = [
    lambda: t_ffn.test_scalar_hand_case(),
    lambda: t_ffn.test_dense_matches_numpy_matmul(1, 40, 24, 2),
    lambda: t_ffn.test_prefix_matches_numpy(4, 24, 40, 7),
    lambda: t_ffn.test_neuron_magnitude_is_frobenius_norm_of_rank_one_term(),
    lambda: t_ffn.test_tau_zero_is_dense_bitwise_and_tau_inf_is_zero(),
    lambda: t_ffn.test_brute_force_all_masks_8_neuron_toy(11),
    lambda: t_ffn.test_tie_is_kept_and_strictly_below_is_cut(),
    lambda: t_ffn.test_masks_nested_and_output_is_dense_minus_cut_terms(),
    lambda: t_ffn.test_decode_given_mask_matches_subset_sum(),
]
SIGNAL_PINS = [
    lambda: t_sig.test_closed_form_fixture(),
    lambda: t_sig.test_uniform_is_log_v(1000),
    lambda: t_sig.test_two_point_closed_form(),
    lambda: t_sig.test_matches_scipy_log_softmax_and_pure_python(),
    lambda: t_sig.test_expected_surprisal_is_entropy(),
    lambda: t_sig.test_threshold_truth_table_fixture(),
    lambda: t_sig.test_threshold_layout_signed_coefficients_and_ablation(),
    lambda: t_sig.test_calibrate_is_nearest_rank_order_statistic(10, 0.4),
    lambda: t_sig.test_calibrate_is_nearest_rank_order_statistic(999, 0.3),
]
CETT_PINS = [
    lambda: t_cett.test_worked_example(),
    lambda: t_cett.test_against_pure_python_brute_force(0),
    lambda: t_cett.test_equals_dense_minus_sparse_decode(),
    lambda: t_cett.test_closed_form_for_orthogonal_output_rows(),
    lambda: t_cett.test_limits_and_zero_output_token(),
    lambda: t_cett.test_search_takes_the_last_feasible_candidate_not_the_first_crossing(),
]
MASK_PINS = [
    lambda: t_mask.test_threshold_hand_case(),
    lambda: t_mask.test_threshold_matches_numpy(),
    lambda: t_mask.test_topk_hand_cases(),
    lambda: t_mask.test_topk_matches_numpy_and_python(0),
]
GEGLU_PINS = [
    lambda: t_geglu.test_sigma_values_closed_forms(),
    lambda: t_geglu.test_matches_library_gelu(0),
    lambda: t_geglu.test_limits_and_brute_force_masks(),
    lambda: t_geglu.test_cett_with_gelu_sigma(),
    lambda: t_geglu.test_sigma_argument_does_not_leak_between_calls(),
]
RELU_PINS = [
    lambda: t_relu.test_hand_case(),
    lambda: t_relu.test_matches_numpy(0),
    lambda: t_relu.test_prefix_stats_match_numpy_and_the_decode_function(),
]

RELU_CETT_PINS = [
    lambda: t_relu.test_cett_hand_case(),
    lambda: t_relu.test_cett_is_dense_minus_sparse_over_dense_and_search_is_brute_force(0),
    lambda: t_relu.test_cett_search_takes_the_last_feasible_value_not_the_first_crossing(),
]

# (what is planted, text to find, replacement, pins that must notice)
MUTATIONS = [
    ("ReLU CETT denominator without the output bias",
     "            double f = full[i] + (b_out ? (double)b_out[i] : 0.0);\n            nc += cut[i] * cut[i];",
     "            double f = full[i];\n            nc += cut[i] * cut[i];", RELU_CETT_PINS),
    ("ReLU CETT cut not strict", "            int is_cut = a < eps;", "            int is_cut = a <= eps;", RELU_CETT_PINS),
    ("ReLU CETT numerator carries the output bias",
     "                if (is_cut) cut[i] += n;\n            }\n        }\n        double nc = 0.0, nf = 0.0;\n        for (int i = 0; i < d; ++i) {\n            double f = full[i] + (b_out",
     "                if (is_cut) cut[i] += n;\n            }\n        }\n        double nc = 0.0, nf = 0.0;\n        for (int i = 0; i < d; ++i) {\n            cut[i] += (b_out ? (double)b_out[i] : 0.0);\n            double f = full[i] + (b_out", RELU_CETT_PINS),
    ("ReLU CETT search stops at the first infeasible candidate",
     "        if (m <= bound) { found = 1; best = v; best_mean = m; }\n        while (k < n_ev && ev[k].v == v) {\n            int t = ev[k].t, j = ev[k].j;\n            const float *wo",
     "        if (m <= bound) { found = 1; best = v; best_mean = m; } else if (found) break;\n        while (k < n_ev && ev[k].v == v) {\n            int t = ev[k].t, j = ev[k].j;\n            const float *wo", RELU_CETT_PINS),
    ("ReLU CETT search denominator without the bias",
     "            double f = full[i] + (b_out ? (double)b_out[i] : 0.0);\n            nf += f * f;\n            full[i] = 0.0;",
     "            double f = full[i];\n            nf += f * f;\n            full[i] = 0.0;", RELU_CETT_PINS),
    ("SiLU with the exponent's sign flipped",
     "return g / (1.0 + exp(-g));", "return g / (1.0 + exp(g));", FFN_PINS),
    ("up-projection factor dropped in the decode path",
     "            h[j] = a * u;", "            h[j] = a;", FFN_PINS),
    ("up-projection factor dropped in the prefill path",
     "            double hv = a * u;\n            double aa = fabs(a);", "            double hv = a;\n            double aa = fabs(a);", FFN_PINS),
    ("keep rule strict instead of >=",
     "(fabs(a[(size_t)b * d_ff + j]) >= tau[b]) ? 1 : 0;", "(fabs(a[(size_t)b * d_ff + j]) > tau[b]) ? 1 : 0;", FFN_PINS),
    ("magnitude dropped from the keep rule",
     "(fabs(a[(size_t)b * d_ff + j]) >= tau[b]) ? 1 : 0;", "(a[(size_t)b * d_ff + j] >= tau[b]) ? 1 : 0;", FFN_PINS),
    ("output row read back to front",
     "                for (int i = lo; i < hi; ++i) yb[i] += hv * (double)wd[i];",
     "                for (int i = lo; i < hi; ++i) yb[i] += hv * (double)wd[d - 1 - i];", FFN_PINS),
    ("A_j without the square root of the summed squares",
     "if (A) A[j] = sqrt(s_h2) * sqrt(wn2);\n    }\n    if (y) {\n#pragma omp parallel for schedule(static)\n        for (int t = 0; t < T; ++t) {\n            double *yt = y + (size_t)t * d;\n            for (int i = 0; i < d; ++i) yt[i] = 0.0;\n            for (int j = 0; j < d_ff; ++j) {\n                double hv = h[(size_t)t * d_ff + j];\n                const float *wd",
     "if (A) A[j] = s_h2 * sqrt(wn2);\n    }\n    if (y) {\n#pragma omp parallel for schedule(static)\n        for (int t = 0; t < T; ++t) {\n            double *yt = y + (size_t)t * d;\n            for (int i = 0; i < d; ++i) yt[i] = 0.0;\n            for (int j = 0; j < d_ff; ++j) {\n                double hv = h[(size_t)t * d_ff + j];\n                const float *wd", FFN_PINS),
    ("sum of |a| accumulates the signed activation",
     "            s_abs += aa;\n            s_sq += a * a;\n            if (aa != aa)", "            s_abs += a;\n            s_sq += a * a;\n            if (aa != aa)", FFN_PINS),
    ("entropy with the wrong sign",
     "if (p > 0.0) H -= p * logp;", "if (p > 0.0) H += p * logp;", SIGNAL_PINS),
    ("surprisal measured from the maximum instead of the log-sum-exp",
     "? lse - (double)z[tok[b]] : NAN;", "? m - (double)z[tok[b]] : NAN;", SIGNAL_PINS),
    ("partition function without the max shift undone",
     "double lse = m + log(Z);", "double lse = log(Z);", SIGNAL_PINS),
    ("lambda and gamma attached to the wrong indicators",
     "(1.0 + lambda[l] * is + gamma[l] * ih);", "(1.0 + lambda[l] * ih + gamma[l] * is);", SIGNAL_PINS),
    ("indicator not strict",
     "double is = surprisal[b] > tau_s ? 1.0 : 0.0;", "double is = surprisal[b] >= tau_s ? 1.0 : 0.0;", SIGNAL_PINS),
    ("quantile rank rounded down",
     "double r = ceil((double)q * (double)n);", "double r = floor((double)q * (double)n);", SIGNAL_PINS),
    ("quantile taken one element too high",
     "*tau_base = tmp[clada_oracle_quantile_rank(n, q) - 1];", "*tau_base = tmp[clada_oracle_quantile_rank(n, q) < n ? clada_oracle_quantile_rank(n, q) : n - 1];", SIGNAL_PINS),
    ("CETT cut set not strict",
     "            int is_cut = fabs(a) < eps;", "            int is_cut = fabs(a) <= eps;", CETT_PINS),
    ("CETT ratio of squared norms",
     "cett[t] = nf > 0.0 ? sqrt(nc) / sqrt(nf) : 0.0;", "cett[t] = nf > 0.0 ? nc / nf : 0.0;", CETT_PINS),
    ("CETT search stops at the first infeasible candidate",
     "        if (m <= bound) { found = 1; best = v; best_mean = m; }",
     "        if (m <= bound) { found = 1; best = v; best_mean = m; } else if (found) break;", CETT_PINS),
    ("CETT search bound test strict",
     "        if (m <= bound) { found = 1; best = v; best_mean = m; }",
     "        if (m < bound) { found = 1; best = v; best_mean = m; }", CETT_PINS),
    ("static threshold mask strict",
     "        int keep = A[j] >= tau;", "        int keep = A[j] > tau;", MASK_PINS),
    ("top-k ties to the higher index",
     "    return (x->j > y->j) - (x->j < y->j);               /* then lower index first */",
     "    return (x->j < y->j) - (x->j > y->j);", MASK_PINS),
    ("top-k keeps the smallest scores",
     "if (!xn && x->s != y->s) return (x->s < y->s) - (x->s > y->s);", "if (!xn && x->s != y->s) return (x->s > y->s) - (x->s < y->s);", MASK_PINS),
    ("ReLU FFN without the input bias",
     "double g = dot_fd(w_in + (size_t)j * d, xb, d) + (b_in ? (double)b_in[j] : 0.0);",
     "double g = dot_fd(w_in + (size_t)j * d, xb, d);", RELU_PINS),
    ("ReLU FFN without the output bias",
     "            yb[i] = s + (b_out ? (double)b_out[i] : 0.0);", "            yb[i] = s;", RELU_PINS),
    ("GELU's cubic coefficient off by a factor of ten",
     "(g + 0.044715 * g * g * g)", "(g + 0.44715 * g * g * g)", GEGLU_PINS),
    ("GELU without the factor one half",
     "return 0.5 * g * (1.0 + tanh(", "return g * (1.0 + tanh(", GEGLU_PINS),
    ("GELU with 1 - tanh",
     "return 0.5 * g * (1.0 + tanh(", "return 0.5 * g * (1.0 - tanh(", GEGLU_PINS),
    ("sigma selector ignored: SiLU whatever is asked for",
     "return g_sigma == 1 ? gelu_tanh(g) : silu(g);", "return silu(g);", GEGLU_PINS),
    ("ReLU replaced by the identity",
     "            double v = g > 0.0 ? g : (g != g ? g : 0.0);          /* NaN stays NaN */", "            double v = g;", RELU_PINS),
]


def _load_mutant(path):
    lib = C.CDLL(path)
    lib.clada_oracle_quantile_rank.restype = C.c_int64
    lib.clada_oracle_quantile_rank.argtypes = [C.c_int64, C.c_float]
    return lib


@pytest.mark.parametrize("what,find,repl,pins", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, what, find, repl, pins):
    text = open(SRC).read()
    assert text.count(find) >= 1, f"pattern for '{what}' not found in the oracle source"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(find, repl, 1))
    so = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-std=c99", "-O1", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-w",
                    "-o", str(so), str(src), "-lm"], check=True)
    oracle._load()                                   # make sure the real one is there to restore
    real = oracle._lib
    oracle._lib = _load_mutant(str(so))
    try:
        caught = 0
        for pin in pins:
            try:
                pin()
            except AssertionError:
                caught += 1
        assert caught >= 1, f"no pin noticed: {what}"
    finally:
        oracle._lib = real


def test_unmutated_oracle_passes_every_pin_used_above():
    for pins in (FFN_PINS, SIGNAL_PINS, CETT_PINS, MASK_PINS, RELU_PINS, GEGLU_PINS, RELU_CETT_PINS):
        for pin in pins:
            pin()


# ---- the stored-mask formats (oracle/mask_codec.py, plain Python): the same game on its source text
import importlib.util
import types

import test_oracle_mask_codec as t_codec

CODEC_SRC = os.path.join(os.path.dirname(oracle.__file__), "mask_codec.py")
CODEC_PINS = [
    lambda: t_codec.test_hand_worked_example(),
    lambda: t_codec.test_bit_mask_is_numpy_packbits_and_round_trips(1376, 0.6),
    lambda: t_codec.test_sparse_form_round_trips_and_matches_its_definition(300, 0.5, 0.02),
    lambda: t_codec.test_sparse_form_round_trips_and_matches_its_definition(262144, 0.3, 0.0002),
    lambda: t_codec.test_worst_case_length_bound_is_attained_only_by_wide_gaps(),
]
CODEC_MUTATIONS = [
    ("bit order inside a word reversed", "words[j // 32] |= 1 << (j % 32)", "words[j // 32] |= 1 << (31 - j % 32)"),
    ("gap not reduced by one", "gap = j - prev - 1", "gap = j - prev"),
    ("first gap measured from position 0 instead of -1", "    prev = -1\n    n = 0", "    prev = 0\n    n = 0"),
    ("high group first", "out.append((gap & 127) | 128)\n                gap >>= 7\n            out.append(gap)",
     "out.append((gap >> 7) | 128)\n                gap &= 127\n            out.append(gap)"),
    ("continuation bit on the last byte instead of the others", "out.append((gap & 127) | 128)", "out.append(gap & 127)"),
    ("groups of 8 bits", "gap >>= 7", "gap >>= 8"),
    ("decoder forgets the reference", "words = [int(w) for w in ref_words] if ref_words is not None else [0] * mask_words(d_ff)",
     "words = [0] * mask_words(d_ff)"),
    ("decoder sets instead of flips", "words[pos // 32] ^= 1 << (pos % 32)", "words[pos // 32] |= 1 << (pos % 32)"),
    ("decoder shifts groups by 8", "shift += 7", "shift += 8"),
    ("encoder compares with the mask itself", "if bit != ref:", "if bit:"),
]


@pytest.mark.parametrize("what,find,repl", CODEC_MUTATIONS, ids=[m[0] for m in CODEC_MUTATIONS])
def test_planted_mistake_in_the_mask_codec_is_caught(what, find, repl):
    text = open(CODEC_SRC).read()
    assert text.count(find) >= 1, f"pattern for '{what}' not found"
    mutant = types.ModuleType("mask_codec_mutant")
    exec(compile(text.replace(find, repl, 1), "mask_codec_mutant.py", "exec"), mutant.__dict__)
    real = t_codec.mc
    t_codec.mc = mutant
    try:
        caught = 0
        for pin in CODEC_PINS:
            try:
                pin()
            except (AssertionError, IndexError, ValueError):
                caught += 1
        assert caught >= 1, f"no pin noticed: {what}"
    finally:
        t_codec.mc = real


def test_unmutated_mask_codec_passes_its_pins():
    for pin in CODEC_PINS:
        pin()
