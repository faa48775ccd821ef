"""Planted-mistake check of the pins themselves, entirely on the CPU.

Each mutation is a plausible slip in oracle/hsadmm_oracle.c.  The mutated source is compiled to a
temporary library, swapped in for the oracle, and the pin tests are re-run in-process: at least one of
them must fail.  The mistakes are planted in the oracle only; nothing here touches the GPU path.
"""
import ctypes
import os
import subprocess

import pytest

import oracle
from tests import test_oracle_pins as pins
from tests import test_oracle_frozen as fpins
from tests import test_oracle_weighted as wpins
from tests import test_oracle_residuals as rpins
from tests import test_oracle_composite as cpins
from tests import test_oracle_shape as spins
from tests import test_oracle_global as gpins
from tests import test_oracle_penalties as ppins
from tests import test_oracle_stopping as tpins
from tests import test_oracle_nested as npins

MUTATIONS = [
    ("tie_goes_to_higher_index", "(kl[h] == kl[g] && h < g)", "(kl[h] == kl[g] && h > g)"),
    ("ties_ignored", "kl[h] > kl[g] || (kl[h] == kl[g] && h < g)", "kl[h] > kl[g]"),
    ("keeps_smallest", "if (kl[h] > kl[g] ||", "if (kl[h] < kl[g] ||"),
    ("keeps_k_plus_one", "ml[g] = before < kk ? 1 : 0;", "ml[g] = before <= kk ? 1 : 0;"),
    ("channel_index_transposed", "v[(o * ci + g) * s + t]", "v[(g * co + o) * s + t]"),
    ("channel_of_element_wrong", "g = (e / s) % ci;", "g = (e % (ci * s)) % ci;"),
    ("dual_regrouped", "U[off + e] = U[off + e] + (wbar[e] - z);", "U[off + e] = (U[off + e] + wbar[e]) - z;"),
    ("dual_sign", "U[off + e] = U[off + e] + (wbar[e] - z);", "U[off + e] = U[off + e] - (wbar[e] - z);"),
    ("mean_by_division", "wbar[e] = acc * inv_R;", "wbar[e] = acc / (float)R;"),
    ("mean_drops_last_replica", "for (int32_t r = 1; r < R; ++r) acc", "for (int32_t r = 1; r < R - 1; ++r) acc"),
    ("candidate_drops_dual", "v[e] = wbar[e] + U[off + e];", "v[e] = wbar[e];"),
    ("key_in_fp32", "const double x = (double)v[g * gs + t];\n                    acc += x * x;",
     "const float x = v[g * gs + t];\n                    acc += (double)(x * x);"),
    ("key_is_abs_sum", "const double x = (double)v[g * gs + t];\n                    acc += x * x;",
     "const double x = (double)v[g * gs + t];\n                    acc += fabs(x);"),
    ("pack_transposed", "pl[(p * n_in + q) * s + t] = sl[", "pl[(q * n_out + p) * s + t] = sl["),
    ("pack_align_ignored", "pos = (pos + pack_align - 1) / pack_align * pack_align;\n        layer_off[l + 1] = pos;",
     "layer_off[l + 1] = pos;"),
    ("expand_no_zero_fill", "for (int64_t e = 0; e < n; ++e) dl[e] = 0.0f;", "for (int64_t e = 0; e < 0; ++e) dl[e] = 0.0f;"),
    ("none_layer_is_pruned", "if (mode[l] == ORACLE_NONE) {\n            for (int64_t g = 0; g < G; ++g) ml[g] = 1;",
     "if (0) {\n            for (int64_t g = 0; g < G; ++g) ml[g] = 1;"),
    ("frozen_mask_inverted", "int keep = mode[l] == ORACLE_NONE || ml[g] != 0;", "int keep = mode[l] == ORACLE_NONE || ml[g] == 0;"),
    ("frozen_ignores_mode_none", "int keep = mode[l] == ORACLE_NONE || ml[g] != 0;", "int keep = ml[g] != 0;"),
    ("frozen_channel_group_wrong", "else if (mode[l] == ORACLE_CHANNEL) g = (e / s) % ci;\n            else g = e / (ci * s);\n            int keep",
     "else if (mode[l] == ORACLE_CHANNEL) g = e % ci;\n            else g = e / (ci * s);\n            int keep"),
    ("frozen_dual_regrouped", "U[off + e] = U[off + e] + (wbar - z);\n            if (Wbar) Wbar[off + e] = wbar;\n        }\n        if (bad)",
     "U[off + e] = (U[off + e] + wbar) - z;\n            if (Wbar) Wbar[off + e] = wbar;\n        }\n        if (bad)"),
    ("frozen_multiplies_by_mask", "const float z = keep ? v : 0.0f;\n            Z[off + e] = z;\n            U[off + e] = U[off + e] + (wbar - z);\n            if (Wbar) Wbar[off + e] = wbar;\n        }\n        if (bad)",
     "const float z = v * (float)keep;\n            Z[off + e] = z;\n            U[off + e] = U[off + e] + (wbar - z);\n            if (Wbar) Wbar[off + e] = wbar;\n        }\n        if (bad)"),
    ("mask_or_is_and", "uint8_t any = 0;\n        for (int32_t i = 0; i < M; ++i) any |= masks[i][g] != 0 ? 1 : 0;",
     "uint8_t any = 1;\n        for (int32_t i = 0; i < M; ++i) any &= masks[i][g] != 0 ? 1 : 0;"),
    ("mask_or_keeps_raw_bytes", "any |= masks[i][g] != 0 ? 1 : 0;", "any |= masks[i][g];"),
    ("weighted_gamma_drops_lambda", "const double gamma = lambda / (double)M + (double)P * rho1[l] + rho2[l];", "const double gamma = (double)P * rho1[l] + rho2[l];"),
    ("weighted_gamma_forgets_P", "const double gamma = lambda / (double)M + (double)P * rho1[l] + rho2[l];", "const double gamma = lambda / (double)M + rho1[l] + rho2[l];"),
    ("weighted_lambda_not_divided", "const double gamma = lambda / (double)M +", "const double gamma = lambda +"),
    ("weighted_q_sign", "const float q = Zg[off + e] - Vd[off + e];", "const float q = Zg[off + e] + Vd[off + e];"),
    ("weighted_drops_dual_in_t", "const float t = wbar[e] + U[off + e];\n            const float q", "const float t = wbar[e];\n            const float q"),
    ("weighted_swaps_coefficients", "const float at = al * t;\n            const float bq = bl * q;", "const float at = bl * t;\n            const float bq = al * q;"),
    ("weighted_dual_uses_candidate", "const float at = al * t;", "const float at = al * t; wbar[e] = t;"),
    ("dual_inter_sign", "Vd[off + e] = Vd[off + e] + (Zi[off + e] - Zg[off + e]);", "Vd[off + e] = Vd[off + e] + (Zg[off + e] - Zi[off + e]);"),
    ("add_arenas_subtracts", "C[off + e] = A[off + e] + B[off + e];", "C[off + e] = A[off + e] - B[off + e];"),
    ("residual_in_fp32", "const double d = (double)W[r][off + e] - zi;", "const double d = (double)(W[r][off + e] - (float)zi);"),
    ("residual_skips_a_replica", "for (int32_t r = 0; r < R; ++r) {\n                const double d = (double)W[r][off + e] - zi;", "for (int32_t r = 1; r < R; ++r) {\n                const double d = (double)W[r][off + e] - zi;"),
    ("residual_abs_not_square", "const double d = zi - (double)Zi_prev[off + e]; s_in += d * d;", "const double d = zi - (double)Zi_prev[off + e]; s_in += fabs(d);"),
    ("residual_rows_swapped", "out[1 * (int64_t)L + l] = s_in;\n        out[2 * (int64_t)L + l] = r_out;", "out[2 * (int64_t)L + l] = s_in;\n        out[1 * (int64_t)L + l] = r_out;"),
    ("residual_inter_dual_uses_zi", "const double d = (double)Zg[off + e] - (double)Zg_prev[off + e]; s_out += d * d;", "const double d = zi - (double)Zg_prev[off + e]; s_out += d * d;"),
    ("filter_mask_prunes_channels_too", "if ((mode != ORACLE_CHANNEL && mode != ORACLE_BOTH) || mc[c]) k_in[b++]", "if (mode == ORACLE_NONE || mc[c % co]) k_in[b++]"),
    ("composite_channels_first", "project_in_place(x, co, ci, s, 0, k_out, key, m);\n    project_in_place(x, co, ci, s, 1, k_in, key + co, m + co);",
     "project_in_place(x, co, ci, s, 1, k_in, key + co, m + co);\n    project_in_place(x, co, ci, s, 0, k_out, key, m);"),
    ("composite_counts_swapped", "project_in_place(x, co, ci, s, 0, k_out, key, m);\n    project_in_place(x, co, ci, s, 1, k_in, key + co, m + co);",
     "project_in_place(x, co, ci, s, 0, k_in, key, m);\n    project_in_place(x, co, ci, s, 1, k_out, key + co, m + co);"),
    ("composite_stage_tie_rule", "(key[h] == key[g] && h < g)", "(key[h] == key[g] && h > g)"),
    ("composite_stage_channel_transposed", "x[(o * ci + g) * s + t]", "x[(g * co + o) * s + t]"),
    ("composite_stage_zeroes_wrong_group", "(channel ? (e / s) % ci : e / (ci * s));", "(channel ? e % ci : e / (ci * s));"),
    ("drift_counts_raw_bytes", "d += ((a[gbase + g] != 0) != (b[gbase + g] != 0)) ? 1 : 0;", "d += (a[gbase + g] != b[gbase + g]) ? 1 : 0;"),
    ("drift_counts_unconstrained_layers", "if (mode[l] != ORACLE_NONE)\n            for (int64_t g = 0; g < G; ++g) d +=", "if (1)\n            for (int64_t g = 0; g < G; ++g) d +="),
    ("average_by_division", "out[e] = acc * inv_M;", "out[e] = acc / (float)M;"),
    ("average_drops_last_node", "for (int32_t i = 1; i < M; ++i) acc = acc + bufs[i][e];", "for (int32_t i = 1; i < M - 1; ++i) acc = acc + bufs[i][e];"),
    ("average_sums_in_double", "float acc = bufs[0][e];\n        for (int32_t i = 1; i < M; ++i) acc = acc + bufs[i][e];", "double acc = bufs[0][e];\n        for (int32_t i = 1; i < M; ++i) acc = acc + bufs[i][e];"),
    ("shape_key_stride_wrong", "const double y = (double)x[o * ci * s + g];", "const double y = (double)x[o * ci + g];"),
    ("shape_zeroes_wrong_group", "const int64_t g = channel == 2 ? e % (ci * s) :", "const int64_t g = channel == 2 ? e % ci :"),
    ("shape_group_count_is_channels", "const int64_t G = channel == 2 ? ci * s : (channel ? ci : co);", "const int64_t G = channel == 2 ? ci : (channel ? ci : co);"),
    ("shape_packed_as_whole_channels", "if (lm == ORACLE_SHAPE) {\n            /* shape groups", "if (0) {\n            /* shape groups"),
    ("shape_frozen_group_wrong", "if (mode[l] == ORACLE_SHAPE) g = e % (ci * s);", "if (mode[l] == ORACLE_SHAPE) g = (e / s) % (ci * s);"),
    ("composite_dual_regrouped", "U[off + e] = U[off + e] + (wbar[e] - v[e]);", "U[off + e] = (U[off + e] + wbar[e]) - v[e];"),
    ("composite_channel_bytes_misplaced", "const uint8_t *mc = mode == ORACLE_BOTH ? ml + co : ml;", "const uint8_t *mc = mode == ORACLE_BOTH ? ml + ci : ml;"),
    ("composite_kept_idx_channels_first", "if (lm != ORACLE_CHANNEL)\n            for (int64_t p = 0; p < n_out; ++p) kept_idx[nk++] = k_out[p];\n        if (lm == ORACLE_CHANNEL || lm == ORACLE_BOTH)\n            for (int64_t q = 0; q < n_in; ++q) kept_idx[nk++] = k_in[q];",
     "if (lm == ORACLE_CHANNEL || lm == ORACLE_BOTH)\n            for (int64_t q = 0; q < n_in; ++q) kept_idx[nk++] = k_in[q];\n        if (lm != ORACLE_CHANNEL)\n            for (int64_t p = 0; p < n_out; ++p) kept_idx[nk++] = k_out[p];"),
    ("composite_frozen_or_instead_of_and", "keep = keep && ml[co + (e / s) % ci] != 0;", "keep = keep || ml[co + (e / s) % ci] != 0;"),
    ("composite_frozen_channel_byte_offset", "keep = keep && ml[co + (e / s) % ci] != 0;", "keep = keep && ml[(e / s) % ci] != 0;"),
    ("composite_weighted_projects_filters_only",
     "return -2; }\n        if (mode[l] >= ORACLE_BOTH) {\n            if (mode[l] == ORACLE_BOTH) project_composite(v, co, ci, s, k[l], k_in[l],",
     "return -2; }\n        if (mode[l] >= ORACLE_BOTH) {\n            if (mode[l] == ORACLE_BOTH) project_composite(v, co, ci, s, k[l], ci,"),
    ("weighted_frozen_drops_global_term", "const float zt = at + bq;", "const float zt = at;"),
    ("weighted_frozen_mask_ignored", "const float z = keep ? zt : 0.0f;", "const float z = zt;"),
    ("weighted_frozen_candidate_drops_dual", "const float t = wbar + U[off + e];", "const float t = wbar;"),
    ("weighted_frozen_dual_uses_unmasked_candidate",
     "const float z = keep ? zt : 0.0f;\n            Z[off + e] = z;\n            U[off + e] = U[off + e] + (wbar - z);",
     "const float z = keep ? zt : 0.0f;\n            Z[off + e] = z;\n            U[off + e] = U[off + e] + (wbar - zt);"),
    ("penalty_rule_inverted", "if (r > mu * s) {\n                next = tau_incr * old;", "if (r < mu * s) {\n                next = tau_incr * old;"),
    ("penalty_cap_ignored", "if (next > cap) next = cap;", "if (next > cap) next = next;"),
    ("penalty_scale_inverted", "[l] = (float)(old / next);", "[l] = (float)(next / old);"),
    ("penalty_dual_norm_without_rho", "const double s = *rho * sqrt(copies *", "const double s = sqrt(copies *"),
    ("penalty_dual_norm_without_copies", "const double s = *rho * sqrt(copies * sq[", "const double s = *rho * sqrt(sq["),
    ("penalty_reads_the_wrong_rows", "const double r = sqrt(sq[(int64_t)(2 * level) * L + l]);", "const double r = sqrt(sq[(int64_t)(level) * L + l]);"),
    ("penalty_cut_multiplies", "next = old / tau_decr;", "next = old * tau_decr;"),
    ("penalty_compares_squares_with_mu", "const double r = sqrt(sq[(int64_t)(2 * level) * L + l]);", "const double r = sq[(int64_t)(2 * level) * L + l];"),
    ("scale_layers_takes_the_first_factor", "const float f = factor[l];", "const float f = factor[0];"),
    ("stop_primal_not_strict", "done[l] = (r_pri < eps_pri && r_dual < eps_dual) ? 1 : 0;", "done[l] = (r_pri <= eps_pri && r_dual < eps_dual) ? 1 : 0;"),
    ("stop_dual_not_strict", "done[l] = (r_pri < eps_pri && r_dual < eps_dual) ? 1 : 0;", "done[l] = (r_pri < eps_pri && r_dual <= eps_dual) ? 1 : 0;"),
    ("stop_either_side_suffices", "done[l] = (r_pri < eps_pri && r_dual < eps_dual) ? 1 : 0;", "done[l] = (r_pri < eps_pri || r_dual < eps_dual) ? 1 : 0;"),
    ("stop_takes_the_smaller_stack", "eps_rel * (ax > bz ? ax : bz);", "eps_rel * (ax < bz ? ax : bz);"),
    ("stop_dual_norm_forgets_P", "const double r_dual = sqrt((double)P * rho1[l] * rho1[l] * sq[1 * (int64_t)L + l] +", "const double r_dual = sqrt(rho1[l] * rho1[l] * sq[1 * (int64_t)L + l] +"),
    ("stop_dual_norm_rho_not_squared", "const double r_dual = sqrt((double)P * rho1[l] * rho1[l] * sq[1 * (int64_t)L + l] +", "const double r_dual = sqrt((double)P * rho1[l] * sq[1 * (int64_t)L + l] +"),
    ("stop_primal_drops_inter_level", "const double r_pri = sqrt(sq[0 * (int64_t)L + l] + sq[2 * (int64_t)L + l]);", "const double r_pri = sqrt(sq[0 * (int64_t)L + l]);"),
    ("stop_scaled_duals_in_threshold", "const double aty = sqrt(rho1[l] * rho1[l] * mag[3 * (int64_t)L + l] + rho2[l] * rho2[l] * mag[4 * (int64_t)L + l]);", "const double aty = sqrt(mag[3 * (int64_t)L + l] + mag[4 * (int64_t)L + l]);"),
    ("stop_dimension_forgets_the_inter_block", "const double p = (double)(P + 1) * (double)n_elems[l] * (double)n_out;", "const double p = (double)P * (double)n_elems[l] * (double)n_out;"),
    ("stop_bz_forgets_copies_of_zi", "const double bz = sqrt((double)P * mag[1 * (int64_t)L + l] +", "const double bz = sqrt(mag[1 * (int64_t)L + l] +"),
    ("stop_overall_flag_is_any", "if (!done[l]) every = 0;", "if (done[l]) every = 1; else if (l == 0) every = 0;"),
    ("layer_sqnorm_in_fp32", "const double x = (double)X[off + e];\n            s += x * x;", "const float x = X[off + e];\n            s += (double)(x * x);"),
    ("nested_ranks_positions_of_pruned_channels", "if (cm[h / s] && (key[h] > key[g] ||", "if ((key[h] > key[g] ||"),
    ("nested_keeps_positions_of_pruned_channels", "if (!cm[g / s]) { m[g] = 0; continue; }", "if (0) { m[g] = 0; continue; }"),
    ("nested_channel_of_position_wrong", "if (!cm[g / s]) { m[g] = 0; continue; }", "if (!cm[g % ci]) { m[g] = 0; continue; }"),
    ("nested_tie_rule", "(key[h] > key[g] || (key[h] == key[g] && h < g))) ++before;", "(key[h] > key[g] || (key[h] == key[g] && h > g))) ++before;"),
    ("nested_shape_key_stride_wrong", "const double y = (double)x[o * G + g];", "const double y = (double)x[o * ci + g];"),
    ("nested_shapes_before_channels", "    project_in_place(x, co, ci, s, 1, k_in, key, m);\n    project_shapes_within(x, co, ci, s, k_kern, m, key + ci, m + ci);",
     "    for (int64_t c = 0; c < ci; ++c) m[c] = 1;\n    project_shapes_within(x, co, ci, s, k_kern, m, key + ci, m + ci);\n    project_in_place(x, co, ci, s, 1, k_in, key, m);"),
    ("nested_filters_skipped", "    if (filters) {\n        project_in_place(x, co, ci, s, 0, k_out, key, m);", "    if (filters) {\n        project_in_place(x, co, ci, s, 0, co, key, m);"),
    ("nested_counts_swapped", "project_shapes_within(x, co, ci, s, k_kern, m, key + ci, m + ci);\n}", "project_shapes_within(x, co, ci, s, k_in, m, key + ci, m + ci);\n}"),
    ("nested_zeroes_wrong_position", "if (!m[e % G]) x[e] = 0.0f;", "if (!m[e / co % G]) x[e] = 0.0f;"),
    ("nested_weighted_takes_the_base_candidate_counts", "else project_nested(v, co, ci, s, mode[l] == ORACLE_ALL, k[l], k_in[l], k_kern[l], key + gbase, mask + gbase);\n#pragma omp parallel for schedule(static)\n            for (int64_t e = 0; e < n; ++e) {\n                Z[off + e] = v[e];\n                U[off + e] = U[off + e] + (wbar[e] - v[e]);\n                if (Wbar) Wbar[off + e] = wbar[e];\n            }\n            free(wbar);\n            free(v);\n            gbase += G;\n            continue;\n        }\n        double *kl = key + gbase;\n#pragma omp parallel for schedule(static)\n        for (int64_t g = 0; g < G; ++g) {\n            double acc = 0.0;\n            if (mode[l] == ORACLE_CHANNEL) {",
     "else project_nested(v, co, ci, s, mode[l] == ORACLE_ALL, k[l], ci, k_kern[l], key + gbase, mask + gbase);\n#pragma omp parallel for schedule(static)\n            for (int64_t e = 0; e < n; ++e) {\n                Z[off + e] = v[e];\n                U[off + e] = U[off + e] + (wbar[e] - v[e]);\n                if (Wbar) Wbar[off + e] = wbar[e];\n            }\n            free(wbar);\n            free(v);\n            gbase += G;\n            continue;\n        }\n        double *kl = key + gbase;\n#pragma omp parallel for schedule(static)\n        for (int64_t g = 0; g < G; ++g) {\n            double acc = 0.0;\n            if (mode[l] == ORACLE_CHANNEL) {"),
    ("layer_sqnorm_reads_padding", "for (int64_t e = 0; e < n; ++e) {\n            const double x = (double)X[off + e];", "for (int64_t e = 0; e < n + 1; ++e) {\n            const double x = (double)X[off + e];"),
]

PIN_FUNCS = [
    lambda: [pins.test_handworked_layer(c) for c in pins.CASES],
    pins.test_handworked_two_layer_offsets_and_alignment,
    lambda: [pins.test_projection_is_the_euclidean_projection_by_brute_force(m, 0) for m in (1, 2)],
    lambda: [pins.test_against_numpy_library_routines(s) for s in range(3)],
    pins.test_compact_takes_an_arbitrary_source_and_mask,
    pins.test_ties_identical_groups_resolve_by_lower_index,
    pins.test_dual_update_parenthesisation_of_eq_12,
    pins.test_mean_is_left_to_right_sum_times_reciprocal,
    pins.test_eq_9_reduces_to_plain_mean_plus_mean_dual,
    pins.test_invariants_on_tiny_and_random_workloads,
    pins.test_identity_cases,
    fpins.test_handworked_frozen_masks,
    lambda: [fpins.test_frozen_with_the_projections_own_mask_is_the_projection(s) for s in range(2)],
    lambda: [fpins.test_frozen_against_the_printed_formula_in_numpy(s) for s in range(2)],
    fpins.test_all_ones_mask_and_unconstrained_layers,
    fpins.test_mask_union_is_the_logical_or,
    fpins.test_mask_drift_counts_changed_groups_per_layer,
    wpins.test_coefficients_of_eq_9,
    wpins.test_handworked_weighted_projection,
    lambda: [wpins.test_weights_one_and_zero_give_the_base_projection(s) for s in range(2)],
    wpins.test_eq_9_printed_formula_with_per_replica_duals,
    lambda: [wpins.test_weighted_against_numpy(s) for s in range(2)],
    wpins.test_inter_node_dual_update_and_transmission_sum,
    lambda: [wpins.test_weighted_frozen_with_its_own_mask_is_the_dynamic_weighted_projection(s) for s in range(2)],
    lambda: [wpins.test_weighted_frozen_with_weights_one_and_zero_is_the_base_frozen_projection(s) for s in range(2)],
    wpins.test_weighted_frozen_against_the_printed_formulas_in_float64,
    rpins.test_handworked_residuals,
    rpins.test_residuals_against_numpy_and_their_zero_cases,
    lambda: [cpins.test_handworked_composite_layer(c) for c in cpins.CASES],
    cpins.test_the_selection_depends_on_the_order_and_the_oracle_takes_filters_first,
    lambda: [cpins.test_composite_is_the_two_single_projections_applied_in_sequence(s) for s in range(2)],
    lambda: [cpins.test_composite_against_numpy_library_routines(s) for s in range(2)],
    cpins.test_separable_magnitudes_have_a_closed_form_answer,
    cpins.test_invariants_feasibility_conservation_idempotence,
    cpins.test_frozen_mask_under_both_constraints,
    cpins.test_weighted_candidate_under_both_constraints,
    cpins.test_union_of_composite_masks_packs_the_union_of_both_index_sets,
    gpins.test_handworked_mean_of_node_buffers,
    lambda: [gpins.test_mean_equals_the_pinned_replica_mean_and_numpy(s) for s in range(2)],
    spins.test_handworked_shape_layer,
    lambda: [spins.test_shape_groups_are_the_columns_of_the_gemm_view(s) for s in range(2)],
    lambda: [spins.test_shape_against_numpy(s) for s in range(2)],
    ppins.test_handworked_balancing_both_levels_and_the_cap,
    ppins.test_the_inequalities_are_strict_and_the_dual_norm_counts_the_copies,
    ppins.test_repeated_raises_follow_the_closed_form_count,
    ppins.test_layers_and_levels_are_independent_and_neutral_constants_change_nothing,
    ppins.test_rescaled_dual_keeps_a_converged_scaled_admm_at_its_fixed_point,
    ppins.test_scale_layers_is_a_per_layer_float32_multiply,
    tpins.test_handworked_thresholds_one_layer,
    tpins.test_both_comparisons_are_strict,
    tpins.test_relative_part_takes_the_larger_of_the_two_stacks_and_the_unscaled_duals,
    tpins.test_the_residual_totals_count_replicas_and_nodes,
    tpins.test_layers_are_judged_separately_and_the_overall_flag_needs_all_of_them,
    tpins.test_against_the_formulas_in_numpy_on_random_inputs,
    tpins.test_layer_sqnorms_handworked_and_against_numpy,
    lambda: [npins.test_handworked_nested_layer(c) for c in npins.CASES],
    lambda: [npins.test_special_cases_reduce_to_the_modes_pinned_elsewhere(s) for s in range(2)],
    lambda: [npins.test_against_the_single_projections_applied_literally_with_numpy(s) for s in range(2)],
    npins.test_the_shape_selection_is_the_best_one_inside_the_kept_channels_by_brute_force,
    npins.test_ties_between_identical_channels_and_positions_go_to_the_lower_index,
    npins.test_weighted_candidate_under_the_nested_modes,
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_in_the_oracle_fails_a_pin(name, old, new, tmp_path, monkeypatch):
    src = open(os.path.join(os.path.dirname(oracle.__file__), "hsadmm_oracle.c")).read()
    assert src.count(old) >= 1, "mutation target not found: %s" % name
    mutated = src.replace(old, new, 1)
    c_file = tmp_path / "mut.c"
    so_file = tmp_path / "libmut.so"
    c_file.write_text(mutated)
    subprocess.check_call(["gcc", *[f for f in oracle.CFLAGS if f not in ("-Wall", "-Wextra")], "-w",
                           "-o", str(so_file), str(c_file), "-lm"])
    good = oracle._load()
    lib = ctypes.CDLL(str(so_file))
    for fn in ("oracle_project", "oracle_compact", "oracle_expand", "oracle_set_threads", "oracle_get_threads",
               "oracle_project_frozen", "oracle_mask_or", "oracle_node_coefficients", "oracle_project_weighted",
               "oracle_dual_inter", "oracle_add_arenas", "oracle_residuals", "oracle_average", "oracle_mask_drift",
               "oracle_project_weighted_frozen", "oracle_adapt_penalties", "oracle_scale_layers", "oracle_layer_sqnorms",
               "oracle_stopping_test"):
        getattr(lib, fn).argtypes = getattr(good, fn).argtypes
        getattr(lib, fn).restype = getattr(good, fn).restype
    monkeypatch.setattr(oracle, "_lib", lib)
    failed = 0
    for f in PIN_FUNCS:
        try:
            f()
        except (AssertionError, ValueError):
            failed += 1
    assert failed >= 1, "no pin noticed the planted mistake %r" % name
