"""Plant plausible mistakes in the oracle (on the CPU, in a temporary copy of its
source) and require that the pins catch every one of them."""
import os
import subprocess

import pytest

import oracle
import oracle_pins

SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "moe_oracle.c")

MUTANTS = {
    "silu_on_up_branch": ("m[f] = (a / (1.0 + exp(-a))) * u;", "m[f] = (u / (1.0 + exp(-u))) * a;"),
    "silu_sign": ("exp(-a)", "exp(a)"),
    "down_transposed": ("w_down[(size_t)h * F + f]", "w_down[(size_t)f * H + h]"),
    "gate_transposed": ("w_gate[(size_t)f * H + h]", "w_gate[(size_t)h * F + f]"),
    "up_reads_gate": ("bf16_to_f64(w_up[", "bf16_to_f64(w_gate["),
    "tie_break_high_id": ("s[e] > s[best]", "s[e] >= s[best]"),
    "slot_zero_is_miss": ("if (slot_table[e] < 0) continue;", "if (slot_table[e] <= 0) continue;"),
    "gate_weight_dropped": ("y[h] += g * o;", "y[h] += o;"),
    "hist_saturates": ("hist[topk_idx[a]] += 1;", "hist[topk_idx[a]] = 1;"),
    "miss_list_holds_expert": ("miss_list[n++] = a;", "miss_list[n++] = topk_idx[a];"),
    "bias_dropped": ("if (bias) s += (double)bias[e];", ""),
    "router_transposed": ("router_w[(size_t)e * H + h]", "router_w[(size_t)h * E + e]"),
    "shared_weight_half": ("1.0, y + (size_t)t * H);", "0.5, y + (size_t)t * H);"),
    "weights_by_slot": ("size_t off = (size_t)e * F * H;", "size_t off = (size_t)slot_table[e] * F * H;"),
    "gate_not_normalised": ("- smax) / den;", "- smax);"),
    "est_downward_test_first": ("if (d >= (int64_t)th_up[i]) {\n            s[i] = s[i] + 1 < K ? s[i] + 1 : K;\n        } else if (-d >= (int64_t)th_dn[i]) {\n            s[i] = s[i] - 1 > 0 ? s[i] - 1 : 0;\n        }",
                                "if (-d >= (int64_t)th_dn[i]) {\n            s[i] = s[i] - 1 > 0 ? s[i] - 1 : 0;\n        } else if (d >= (int64_t)th_up[i]) {\n            s[i] = s[i] + 1 < K ? s[i] + 1 : K;\n        }"),
    "est_strict_upward": ("if (d >= (int64_t)th_up[i]) {", "if (d > (int64_t)th_up[i]) {"),
    "est_no_upper_clamp": ("s[i] = s[i] + 1 < K ? s[i] + 1 : K;", "s[i] = s[i] + 1;"),
    "est_no_lower_clamp": ("s[i] = s[i] - 1 > 0 ? s[i] - 1 : 0;", "s[i] = s[i] - 1;"),
    "est_calibrates_wrong_side": ("th_dn[i] = (int32_t)(((int64_t)(lam_den - lam_num) * th_dn[i]", "th_up[i] = (int32_t)(((int64_t)(lam_den - lam_num) * th_dn[i]"),
    "est_floor_becomes_round": ("+ (int64_t)lam_num * d) / lam_den);", "+ (int64_t)lam_num * d + lam_den / 2) / lam_den);"),
    "est_lambda_swapped": ("(int64_t)(lam_den - lam_num) * th_up[i] + (int64_t)lam_num * d)", "(int64_t)lam_num * th_up[i] + (int64_t)(lam_den - lam_num) * d)"),
    "est_f_prev_not_kept": ("        f_prev[i] = f[i];\n", ""),
    "est_signed_fluctuation_in_dn": ("(int64_t)lam_num * (-d)) / lam_den);", "(int64_t)lam_num * d) / lam_den);"),
    "prefetch_counts_residents": ("if (s[i] >= tau && slot_table[i] < 0) n += 1;", "if (s[i] >= tau && slot_table[i] >= 0) n += 1;"),
    "prefetch_strict_threshold": ("if (s[i] >= tau && slot_table[i] < 0) n += 1;", "if (s[i] > tau && slot_table[i] < 0) n += 1;"),
    "bal_b_counts_assignments": ("if (f[i] > 0) b += 1;", "if (f[i] > 0) b += f[i];"),
    "bal_cpu_time_uses_b": ("double tc = ((r_c[tau] * (double)gamma) * (double)k) * t_cpu;", "double tc = (r_c[tau] * (double)b) * t_cpu;"),
    "bal_gpu_time_uses_gamma_k": ("double tg = (r_g[tau] * (double)b) * t_gpu;", "double tg = ((r_g[tau] * (double)gamma) * (double)k) * t_gpu;"),
    "bal_window_uses_min": ("double total = tc > tg ? tc : tg;", "double total = tc < tg ? tc : tg;"),
    "bal_draft_term_not_per_layer": ("((double)gamma * t_draft) / (double)l_target;", "((double)gamma * t_draft);"),
    "bal_io_strict": ("<= window;", "< window;"),
    "bal_memory_ignored": ("if (!io_ok || !mem_ok) continue;", "if (!io_ok) continue;"),
    "bal_io_ignored": ("if (!io_ok || !mem_ok) continue;", "if (!mem_ok) continue;"),
    "bal_signed_objective": ("double obj = fabs(tc - tg);", "double obj = tc - tg;"),
    "bal_ties_to_larger": ("if (best < 0 || obj < best_f) {", "if (best < 0 || obj <= best_f) {"),
    "bal_fallback_one": ("return best < 0 ? K : best;", "return best < 0 ? 1 : best;"),
    "bal_tau_from_zero": ("for (int tau = 1; tau <= K; ++tau) {\n        double tc", "for (int tau = 0; tau <= K; ++tau) {\n        double tc"),
    "plan_evicts_frozen": ("if (slot_table[i] >= 0 && !in_use[i] && s[i] == level) evict_list[ne++] = i;", "if (slot_table[i] >= 0 && s[i] == level) evict_list[ne++] = i;"),
    "plan_evicts_at_threshold": ("for (int level = 0; level < tau; ++level)", "for (int level = 0; level <= tau; ++level)"),
    "plan_fetch_low_levels_first": ("for (int level = K; level >= tau && level >= 0; --level) {", "for (int level = tau < 0 ? 0 : tau; level <= K; ++level) {"),
    "plan_fetch_below_threshold": ("for (int level = K; level >= tau && level >= 0; --level) {", "for (int level = K; level >= tau - 1 && level >= 0; --level) {"),
    "plan_ignores_budget": ("            if (nf >= budget) continue;\n", ""),
    "plan_reuses_taken_slot": ("            slot_free[next_slot] = 0;\n            slot_table[i] = next_slot;", "            slot_table[i] = next_slot;"),
    "plan_keeps_evicted_in_table": ("    for (int j = 0; j < ne; ++j) slot_table[evict_list[j]] = -1;\n", ""),
    "plan_refetches_residents": ("if (slot_table[i] >= 0 || s[i] != level) continue;", "if (s[i] != level) continue;"),
    "descending_order_lost": ("topk_idx[(size_t)t * k + j] = best;", "topk_idx[(size_t)t * k + (k - 1 - j)] = best;"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found"
    mutated = text.replace(old, new)
    c = tmp_path / "mutant.c"
    so = tmp_path / "mutant.so"
    c.write_text(mutated)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", str(so), str(c), "-lm"])
    O = oracle.Oracle(str(so))
    caught = []
    for pin in oracle_pins.ALL_PINS:
        try:
            pin(O)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake '{name}'"
