"""Do the pins of the MoE oracle have teeth?  Each case plants one plausible mistake in a copy
of the oracle's source (on the CPU, in a temporary directory), builds it, runs the pins against
the mutant and requires at least one of them to fail.  The unmodified source must pass them all.
Only mistakes that keep every index in bounds are planted: the mutants run in this process."""
import ctypes as C
import os
import subprocess

import pytest

from oracle import ref

import test_oracle_corr_pins as PC
import test_oracle_pins as P
import test_oracle_plan_pins as PP
import test_oracle_q4_pins as PQ

SRC = os.path.join(os.path.dirname(ref.__file__), "moe_oracle.c")

PINS = [P.test_logits_exact_on_small_integers, P.test_logits_within_fp32_bound_of_exact,
        lambda: P.test_logit_order_lane_ownership(4), lambda: P.test_logit_order_lane_ownership(8),
        P.test_topk_bruteforce_with_ties, P.test_topk_duplicate_gate_rows_lower_index_wins,
        P.test_weights_sum_to_one_k1_kE_and_shift, P.test_dispatch_against_stable_sort_and_bruteforce,
        P.test_exec_order_prefers_experts_shared_across_batches, P.test_handworked_layer_fixture,
        P.test_identity_expert_closed_form, P.test_identical_experts_equal_dense_ffn,
        P.test_single_live_expert, P.test_tiny_config_against_dense_numpy_mixture,
        P.test_k_equals_E_is_full_softmax_mixture_with_shared_and_token_subset,
        P.test_bf16_weight_path_matches_float_path, P.test_output_invariant_under_expert_relabelling,
        PC.test_update_matches_histogram2d_and_accumulates, PC.test_update_hand_count,
        PC.test_predict_deterministic_map_recovers_permuted_counts, PC.test_predict_single_row_and_unseen_rows,
        PC.test_predict_uniform_rows_give_equal_scores_and_index_order, PC.test_predict_against_exact_rationals,
        PQ.test_hand_worked_group, PQ.test_matches_numpy_broadcast_and_nibble_order,
        PQ.test_zero_point_code_is_exact_zero_and_integers_stay_integers,
        PQ.test_round_trip_error_is_at_most_half_a_step, PQ.test_double_weights_feed_the_expert_like_float32_ones,
        PQ.test_rounding_to_bf16_matches_the_library_conversion_and_hand_ties,
        PQ.test_dequant_to_original_precision_is_the_rounded_exact_value,
        PP.test_hand_solved_cases, PP.test_result_is_the_smallest_n_that_satisfies_the_group_exactly,
        PP.test_each_inequality_can_be_the_binding_one, PP.test_best_and_worst_case_of_the_paper,
        PP.test_invariances_and_monotonicity]

MUTATIONS = {
    "ties go to the higher index": ("if (best < 0 || row[e] > row[best]) best = e;", "if (best < 0 || row[e] >= row[best]) best = e;"),
    "smallest logits selected": ("if (best < 0 || row[e] > row[best]) best = e;", "if (best < 0 || row[e] < row[best]) best = e;"),
    "logit lanes own single elements": ("int l = (i / V) % KO_LANES;", "int l = i % KO_LANES;"),
    "butterfly starts at 16": ("for (int m = KO_LANES / 2; m >= 1; m >>= 1) {", "for (int m = KO_LANES / 4; m >= 1; m >>= 1) {"),
    "renormalisation over all experts": ("for (int j = 0; j < k; ++j) den += exp((double)row[sel[j]] - m);", "for (int e = 0; e < E; ++e) den += exp((double)row[e] - m);"),
    "weights not normalised": ("w[(size_t)t * k + j] = exp((double)row[sel[j]] - m) / den;", "w[(size_t)t * k + j] = exp((double)row[sel[j]] - m);"),
    "grouping not stable": ("inv_perm[a] = offsets[e] + seen[e];", "inv_perm[a] = offsets[e] + counts[e] - 1 - seen[e];"),
    "batches counted by tokens": ("for (int j = 0; j < k; ++j) seen[idx[(size_t)t * k + j]] = 1;", "for (int j = 0; j < k; ++j) seen[idx[(size_t)t * k + j]] += 1;"),
    "execution order by token count first": ("int q_first = nbatch[q] > nbatch[e] ||\n                          (nbatch[q] == nbatch[e] &&\n                           (counts[q] > counts[e] || (counts[q] == counts[e] && q < e)));",
                                              "int q_first = counts[q] > counts[e] ||\n                          (counts[q] == counts[e] &&\n                           (nbatch[q] > nbatch[e] || (nbatch[q] == nbatch[e] && q < e)));"),
    "execution order ascending": ("int q_first = nbatch[q] > nbatch[e] ||", "int q_first = nbatch[q] < nbatch[e] ||"),
    "silu without the gate": ("static double silu(double z) { return z / (1.0 + exp(-z)); }", "static double silu(double z) { return 1.0 / (1.0 + exp(-z)); }"),
    "silu with the wrong sign": ("static double silu(double z) { return z / (1.0 + exp(-z)); }", "static double silu(double z) { return z / (1.0 + exp(z)); }"),
    "gate and up swapped": ("h[n] = silu(g) * u;", "h[n] = silu(u) * g;"),
    "down projection transposed": ("s += weight_at(w2, wtype, (size_t)m * f + n) * h[n];", "s += weight_at(w2, wtype, (size_t)n * d + m) * h[n];"),
    "routing weight dropped": ("for (int i = 0; i < d; ++i) y[i] += wt * o[i];", "for (int i = 0; i < d; ++i) y[i] += o[i];"),
    "shared experts weighted like routed": ("double wt = j < k ? w[(size_t)t * k + j] : 1.0;", "double wt = w[(size_t)t * k + (j < k ? j : 0)];"),
    "correlation table transposed": ("table[(size_t)idx_prev[(size_t)t * k + a] * E + idx_cur[(size_t)t * k + b]] += 1;", "table[(size_t)idx_cur[(size_t)t * k + b] * E + idx_prev[(size_t)t * k + a]] += 1;"),
    "correlation counts slots pairwise only": ("for (int b = 0; b < k; ++b)\n                table[", "for (int b = a; b <= a; ++b)\n                table["),
    "tendency not normalised by the row": ("const double freq = (double)table[(size_t)p * E + e] / (double)row;", "const double freq = (double)table[(size_t)p * E + e];"),
    "tendency ignores how many tokens sit on an expert": ("score[e] = score[e] + (double)counts_prev[p] * freq;", "score[e] = score[e] + freq;"),
    "prediction ties go to the higher index": ("if (best < 0 || score[e] > score[best]) best = e; /* first index wins ties */", "if (best < 0 || score[e] >= score[best]) best = e;"),
    "nibbles swapped": ("const int code = (c & 1) ? (byte >> 4) : (byte & 15);", "const int code = (c & 1) ? (byte & 15) : (byte >> 4);"),
    "zero point applied after the scale": ("const double v = s * ((double)code - z);", "const double v = s * (double)code - z;"),
    "scale of the neighbouring group": ("const double s = bf16_to_double(s_bf16[(size_t)r * ng + c / group]);\n            const double z = bf16_to_double(z_bf16[(size_t)r * ng + c / group]);\n            const double v", "const double s = bf16_to_double(s_bf16[(size_t)r * ng + (c / group + 1) % ng]);\n            const double z = bf16_to_double(z_bf16[(size_t)r * ng + c / group]);\n            const double v"),
    "quantisation truncates": ("double v = rint(w[(size_t)r * cols + c] / s + z);", "double v = floor(w[(size_t)r * cols + c] / s + z);"),
    "dequantised weight not rounded to bf16": ("out[(size_t)r * cols + c] = to_bf16 ? round_to_bf16(v) : v;", "out[(size_t)r * cols + c] = v;"),
    "planner: gate compute helps the gate transfer": ("if (!(dn * t_c_A >= t_io_G)) continue;", "if (!(dn * (t_c_A + t_c_G) >= t_io_G)) continue;"),
    "planner: one hot expert too few in the third inequality": ("+ t_c_hotE >= t_io_G + (K + 1) * t_io_E)) continue;", "+ t_c_hotE >= t_io_G + K * t_io_E)) continue;"),
    "planner: attention transfer forgotten": ("(K + len_q) * t_io_E + t_io_A)) continue;", "(K + len_q) * t_io_E)) continue;"),
    "planner: queue compute forgotten": ("+ t_c_hotE + sum_q >= t_io_G", "+ t_c_hotE >= t_io_G"),
    "planner: strict inequalities": ("if (!(dn * (t_c_A + t_c_G) >= t_io_G + K * t_io_E)) continue;", "if (!(dn * (t_c_A + t_c_G) > t_io_G + K * t_io_E)) continue;"),
    "planner: empty queue still waits for the cold path": ("if (len_q > 0) {\n            if (!(dn * (t_c_A + t_c_G) + t_c_hotE", "if (len_q >= 0) {\n            if (!(dn * (t_c_A + t_c_G) + t_c_hotE"),
    "last selected expert skipped": ("for (int j = 0; j < k + S; ++j) {\n                int e = j < k ?", "for (int j = (k > 1); j < k + S; ++j) {\n                int e = j < k ?"),
}


def build_variant(tmp_path, name, old, new):
    text = open(SRC).read()
    if old is not None:
        assert text.count(old) == 1, f"mutation '{name}': pattern occurs {text.count(old)} times"
        text = text.replace(old, new)
    src = tmp_path / "mutant.c"
    lib = tmp_path / "libmutant.so"
    src.write_text(text)
    subprocess.run(["gcc", "-O2", "-mfma", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-o",
                    str(lib), str(src), "-lm"], check=True)
    return C.CDLL(str(lib))


def failures(handle, monkeypatch):
    ref.lib()
    monkeypatch.setattr(ref, "_lib", handle)
    failed = 0
    for pin in PINS:
        try:
            pin()
        except AssertionError:
            failed += 1
    return failed


def test_unmodified_source_passes_every_pin(tmp_path, monkeypatch):
    assert failures(build_variant(tmp_path, "none", None, None), monkeypatch) == 0


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path, monkeypatch):
    old, new = MUTATIONS[name]
    assert failures(build_variant(tmp_path, name, old, new), monkeypatch) >= 1, f"no pin notices: {name}"
