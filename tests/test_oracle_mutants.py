"""The pins of test_oracle_pins.py must be able to SEE a mistake: each plausible slip below
(a wrong sign, a dropped or swapped term, a wrong operand, an off-by-one comparison) is
planted in a copy of the oracle's source, compiled on the CPU, and at least one pin has to
fail on it.  The unmodified source has to pass the same battery.  CPU only."""
import ctypes as C
import os
import subprocess

import pytest

import oracle
import test_oracle_bf16 as half_pins
import test_oracle_loop as loop_pins
import test_oracle_pins as pins
import test_oracle_segments as seg_pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "cocodc_ref.cpp")

# (name, text in cocodc_ref.cpp, replacement); every occurrence is replaced
MUTANTS = [
    ("pseudograd_sign", "static_cast<float>(tg - tm)", "static_cast<float>(tm - tg)"),
    ("momentum_subtracts_grad", "hp.mu * m_old + dg", "hp.mu * m_old - dg"),
    ("momentum_ignores_mu", "hp.mu * m_old + dg", "m_old + dg"),
    ("nesterov_uses_old_momentum", "(dg + hp.mu * m1)", "(dg + hp.mu * m_old)"),
    ("nesterov_drops_mu", "(dg + hp.mu * m1)", "(dg + m1)"),
    ("nesterov_flag_inverted", "hp.nesterov ? (dg + hp.mu * m1) : m1", "hp.nesterov ? m1 : (dg + hp.mu * m1)"),
    ("outer_step_ascends", "theta_g_old - hp.eta * step", "theta_g_old + hp.eta * step"),
    ("outer_step_drops_lr", "theta_g_old - hp.eta * step", "theta_g_old - step"),
    ("drift_operands_swapped", "(theta_send - theta_m);", "(theta_m - theta_send);"),
    ("drift_ignores_sign_switch", "static_cast<double>(hp.drift_sign) * (theta_send - theta_m)", "(theta_send - theta_m)"),
    ("delta_uses_current_params", ": (G - theta_send);", ": (G - theta_m);"),
    ("delta_sign", ": (G - theta_send);", ": (theta_send - G);"),
    ("delta_switch_ignored", "hp.delta_src ? (theta_send - theta_g_prev) : (G - theta_send)", "(G - theta_send)"),
    ("delta_switch_sign", "hp.delta_src ? (theta_send - theta_g_prev)", "hp.delta_src ? (theta_g_prev - theta_send)"),
    ("delta_switch_uses_new_state", "hp.delta_src ? (theta_send - theta_g_prev)", "hp.delta_src ? (theta_send - G)"),
    ("corr_linear_in_d", "hp.lambda * d * d * Delta / tauH", "hp.lambda * d * Delta / tauH"),
    ("corr_divides_by_H_only", "hp.lambda * d * d * Delta / tauH", "hp.lambda * d * d * Delta / static_cast<double>(hp.H)"),
    ("corr_divides_by_tau_only", "hp.lambda * d * d * Delta / tauH", "hp.lambda * d * d * Delta / static_cast<double>(hp.tau)"),
    ("corr_drops_lambda", "hp.lambda * d * d * Delta / tauH", "d * d * Delta / tauH"),
    ("corr_sign", "return G + d + corr;", "return G + d - corr;"),
    ("merge_drops_drift", "return G + d + corr;", "return G + corr;"),
    ("merge_subtracts_drift", "return G + d + corr;", "return G - d + corr;"),
    ("merge_starts_from_local", "return G + d + corr;", "return theta_m + d + corr;"),
    ("blend_weights_swapped", "(1.0 - hp.alpha) * theta_m + hp.alpha * G", "hp.alpha * theta_m + (1.0 - hp.alpha) * G"),
    ("merge_sees_unrounded_global_state", "merge_local(static_cast<double>(G), ts, tm, d, hp, tg)", "merge_local(G64, ts, tm, d, hp, tg)"),
    ("score_sums_values_not_squares", "acc += (norm_kind == 2) ? v * v : std::fabs(v);", "acc += (norm_kind == 2) ? v : std::fabs(v);"),
    ("score_l1_without_abs", "acc += (norm_kind == 2) ? v * v : std::fabs(v);", "acc += (norm_kind == 2) ? v * v : v;"),
    ("score_no_sqrt", "const double norm = (norm_kind == 2) ? std::sqrt(acc) : acc;", "const double norm = acc;"),
    ("score_multiplies_interval", ": norm / static_cast<double>(I_p[p]);", ": norm * static_cast<double>(I_p[p]);"),
    ("score_inf_only_below_zero", "(I_p[p] <= 0) ? std::numeric_limits", "(I_p[p] < 0) ? std::numeric_limits"),
    ("fused_score_no_sqrt", "(hp.norm_kind == 2) ? std::sqrt(s2) : s1", "(hp.norm_kind == 2) ? s2 : s1"),
    ("fused_score_sources_swapped", "const double s2 = hp.score_src ? s.d2 : s.g2;", "const double s2 = hp.score_src ? s.g2 : s.d2;"),
    ("fused_sum_d1_without_abs", "s->d1 += std::fabs(d);", "s->d1 += d;"),
    ("overdue_strict", "t_g - t_b[p] >= static_cast<int64_t>(H)", "t_g - t_b[p] > static_cast<int64_t>(H)"),
    ("overdue_takes_last", "        p_star = p;\n        break;", "        p_star = p;"),
    ("argmax_takes_last_on_tie", "(R[p] > R[p_star])", "(R[p] >= R[p_star])"),
    ("argmin_instead_of_argmax", "(R[p] > R[p_star])", "(R[p] < R[p_star])"),
    ("nan_wins", "std::isnan(R[p_star]) ? !std::isnan(R[p]) : (R[p] > R[p_star])", "(R[p] > R[p_star]) || std::isnan(R[p])"),
    ("selection_with_replacement", "taken[p_star] = 1;", ""),
    ("byte_budget_skips_instead_of_stopping", "if (need > left) break;", "if (need > left) continue;"),
    ("byte_budget_off_by_one", "if (need > left) break;", "if (need >= left) break;"),
    ("planner_min_instead_of_max", "if (cap > static_cast<double>(N))", "if (cap < static_cast<double>(N))"),
    ("planner_ignores_gamma", "std::floor(gamma * ((static_cast<double>(H) * T_c) / T_s))", "std::floor((static_cast<double>(H) * T_c) / T_s)"),
    ("planner_interval_inverted", "static_cast<int64_t>(H) / N;", "N / static_cast<int64_t>(H);"),
    ("event_mask_inverted", "if (!(recv_mask[q] & 1)) continue;", "if (recv_mask[q] & 1) continue;"),
    ("event_mask_ignored", "if (!(recv_mask[q] & 1)) continue;", ""),
    ("event_selects_from_arrived_only", "return select_among(K, R, t_b, t_g, hp->H, budget, in_flight.data(), sel_out, n_sel_out);\n}",
     "for (int32_t q = 0; q < K; ++q) if (!(recv_mask[q] & 1)) R[q] = -1.0;\n  return select_among(K, R, t_b, t_g, hp->H, budget, in_flight.data(), sel_out, n_sel_out);\n}"),
    ("event_ignores_in_flight", "in_flight[q] = (recv_mask[q] & 2) ? 1 : 0;", "in_flight[q] = 0;"),
    ("event_in_flight_bit_confused_with_arrived", "in_flight[q] = (recv_mask[q] & 2) ? 1 : 0;", "in_flight[q] = (recv_mask[q] & 1) ? 1 : 0;"),
    ("f16_truncates", "double q = std::nearbyint(std::ldexp(a, 10 - e));", "double q = std::floor(std::ldexp(a, 10 - e));"),
    ("f16_subnormals_flushed", "if (qi < 1024) return sign | static_cast<uint16_t>(qi);", "if (qi < 1024) return sign;"),
    ("f16_wrong_exponent_bias", "((e + 15) << 10)", "((e + 16) << 10)"),
    ("f16_no_carry_into_the_exponent", "  if (q >= 2048.0) {", "  if (q > 2048.0) {"),
    ("f16_saturates_instead_of_infinity", "    if (e > 15) return sign | 0x7C00;  // 65520 and above round to infinity",
     "    if (e > 15) return sign | 0x7BFF;"),
    ("f16_format_switch_ignored", "return pg_format ? cocodc_ref_round_f16(x) : cocodc_ref_round_bf16(x);",
     "return cocodc_ref_round_bf16(x);"),
    ("half_pg_sign", "round_half(tg - tm, hp.pg_format)", "round_half(tm - tg, hp.pg_format)"),
    ("half_send_record_ignored", "theta_send ? cocodc_ref_widen_bf16(theta_send[i]) : tm;", "tm;"),
    ("half_params_rounded_toward_zero", "theta_m[i] = cocodc_ref_round_bf16(tm_new);",
     "theta_m[i] = cocodc_ref_round_bf16(tm_new); if (std::fabs(cocodc_ref_widen_bf16(theta_m[i])) > std::fabs(tm_new)) theta_m[i] -= 1;"),
    ("half_outer_step_sign", "outer_update(tg, m0, dg, hp, &m1);   // Eq. 2", "outer_update(tg, m0, -dg, hp, &m1);   // Eq. 2"),
    ("half_event_interval_of_fragment_0", "R[q] = score_from_sums(s, I_p[q], *hp);\n    store_sums",
     "R[q] = score_from_sums(s, I_p[0], *hp);\n    store_sums"),
    ("half_sums_stored_for_fragment_0", "store_sums(s, q, sums_out);", "store_sums(s, 0, sums_out);"),
    ("segments_of_every_fragment_walked", "if (segs[j].fragment != p) continue;", ""),
    ("segmented_event_walks_every_shard", "if (segs[j].fragment != q) continue;", ""),
    ("segmented_event_scores_with_interval_of_shard_0", "R[q] = score_from_sums(s, I_p[q], *hp);\n    if (sums_out) {\n      sums_out[4 * q + 0] = s.g2;\n      sums_out[4 * q + 1] = s.g1;\n      sums_out[4 * q + 2] = s.d2;\n      sums_out[4 * q + 3] = s.d1;\n    }\n  }\n  return select_among(K, R, t_b, t_g, hp->H, budget, in_flight.data(), sel_out, n_sel_out);\n}\n\n// ---- bf16",
     "R[q] = score_from_sums(s, I_p[0], *hp);\n    if (sums_out) {\n      sums_out[4 * q + 0] = s.g2;\n      sums_out[4 * q + 1] = s.g1;\n      sums_out[4 * q + 2] = s.d2;\n      sums_out[4 * q + 3] = s.d1;\n    }\n  }\n  return select_among(K, R, t_b, t_g, hp->H, budget, in_flight.data(), sel_out, n_sel_out);\n}\n\n// ---- bf16"),
    ("half_segmented_event_sums_of_shard_0", "store_sums(s, q, sums_out);\n  }\n  return select_among(K, R, t_b, t_g, hp->H, budget, in_flight.data(), sel_out, n_sel_out);\n}\n\n// Eq. 9",
     "store_sums(s, 0, sums_out);\n  }\n  return select_among(K, R, t_b, t_g, hp->H, budget, in_flight.data(), sel_out, n_sel_out);\n}\n\n// Eq. 9"),
    ("in_flight_counts_against_the_budget", "const int32_t n_sel = budget < candidates ? budget : candidates;",
     "const int32_t n_sel = (budget < K ? budget : K) - (K - candidates) > 0 ? (budget < K ? budget : K) - (K - candidates) : 0;"),
]

# (quick pins first: a planted mistake stops the battery at the first pin that sees it)
BATTERY = [
    half_pins.test_f16_rounding_matches_numpy_from_float64_and_torch_from_float32,
    half_pins.test_f16_pseudograd_in_the_bf16_calls,
    lambda ref: loop_pins.test_event_equals_step_on_the_arrived_fragments_then_selection_over_all(ref, (0, 1, 0, 0, 1)),
    lambda ref: seg_pins.test_segmented_event_is_the_segmented_step_on_the_arrived_shards_then_selection(ref, (0, 1, 2, 1)),
    lambda ref: half_pins.test_bf16_segmented_event_is_the_bf16_segmented_step_on_the_arrived_shards_then_selection(ref, (0, 1, 2, 1)),
    half_pins.test_bf16_step_is_the_fp32_step_on_widened_inputs_rounded_once,
    half_pins.test_bf16_segmented_step_against_the_contiguous_and_the_fp32_segmented_steps,
    lambda ref: half_pins.test_bf16_event_is_the_bf16_step_on_the_arrived_fragments_then_selection(ref, (0, 1, 0, 2, 1)),
    pins.test_pseudograd_is_fp32_subtraction_global_minus_local,
    pins.test_pseudograd_sign_and_zero,
    pins.test_unit_outer_step_moves_global_state_to_worker_average,
    pins.test_outer_nesterov_hand_scalar,
    pins.test_outer_without_momentum_is_plain_sgd,
    pins.test_outer_matches_torch_sgd_nesterov,
    pins.test_outer_single_step_from_given_momentum_matches_torch,
    pins.test_delay_compensation_hand_scalar,
    pins.test_zero_delay_reduces_to_adopting_the_global_state,
    pins.test_zero_lambda_gives_no_correction_term,
    pins.test_zero_divergence_gives_no_correction_term,
    pins.test_correction_is_linear_in_lambda,
    pins.test_eq_4_7_8_in_the_papers_own_variables,
    pins.test_change_rate_sign_flip_moves_result_by_twice_the_drift,
    pins.test_single_worker_sync_is_a_no_op_with_reversed_sign,
    pins.test_divergence_term_as_accumulated_local_change,
    pins.test_merge_modes_blend_and_replace,
    pins.test_baseline_merges_need_no_send_time_record,
    pins.test_scores_brute_force_exact_rational,
    pins.test_scores_closed_forms,
    pins.test_score_is_infinite_before_first_sync,
    pins.test_selection_hand_cases,
    pins.test_selection_under_a_byte_budget,
    pins.test_planner_worked_example_from_the_paper,
    pins.test_planner_floor_of_k,
    lambda ref: pins.test_fused_equals_sequence_of_primitives(ref, True),
    pins.test_score_source_and_norm_switches,
    loop_pins.test_selection_passes_over_fragments_in_flight,
    pins.test_selection_exhaustive_small,
]


def _compile(text, path):
    src = path + ".cpp"
    with open(src, "w") as f:
        f.write(text)
    subprocess.run(["g++", "-O1", "-std=c++17", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
                    "-I", os.path.dirname(SRC), "-o", path, src], check=True)
    lib = C.CDLL(path)
    for name in ("pseudograd", "outer_nesterov", "delay_compensate", "fragment_scores", "select_fragments",
                 "sync_step", "sync_step_mt", "sync_plan", "sync_event", "pseudograd_bf16", "sync_step_bf16",
                 "sync_step_segmented", "sync_step_bf16_segmented", "sync_event_bf16", "sync_event_segmented", "sync_event_bf16_segmented"):
        getattr(lib, "cocodc_ref_" + name).restype = C.c_int
    for name, res, arg in (("round_bf16", C.c_uint16, C.c_double), ("widen_bf16", C.c_double, C.c_uint16),
                           ("round_f16", C.c_uint16, C.c_double), ("widen_f16", C.c_double, C.c_uint16)):
        getattr(lib, "cocodc_ref_" + name).restype = res
        getattr(lib, "cocodc_ref_" + name).argtypes = [arg]
    return lib


def _first_failing_pin(lib):
    """Runs the battery against `lib`; returns the name of the first pin that fails, or None."""
    oracle.lib()
    saved = oracle._lib
    oracle._lib = lib
    try:
        for fn in BATTERY:
            try:
                fn(oracle)
            except AssertionError:
                return getattr(fn, "__name__", "fused_equals_sequence")
        return None
    finally:
        oracle._lib = saved


def test_unmodified_oracle_passes_the_battery(tmp_path):
    lib = _compile(open(SRC).read(), str(tmp_path / "clean.so"))
    assert _first_failing_pin(lib) is None


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_every_planted_mistake_is_caught(tmp_path, name, old, new):
    text = open(SRC).read()
    assert old in text, f"mutation site of {name} no longer exists in the oracle source"
    lib = _compile(text.replace(old, new), str(tmp_path / f"{name}.so"))
    caught_by = _first_failing_pin(lib)
    assert caught_by is not None, f"no pin notices the mistake '{name}'"
