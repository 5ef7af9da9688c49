"""The pins must be able to fail: plant one plausible mistake at a time in a copy of the
oracle's C source, build it, and require that the pin tests reject it.  CPU only; the
mistakes are planted in the oracle, never in GPU code."""
import importlib.util
import os
import shutil
import subprocess
import sys

import pytest

import test_oracle_baselines as t_bl
import test_oracle_compact_step as t_cs
import test_oracle_lmhead as t_lm
import test_oracle_score as t_sc
import test_oracle_select as t_se

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sirllm_ref.c")

# (name, text to replace, replacement, pin tests that must catch it)
MUTANTS = [
    ("dropped_token_term", "(m - logit_at(logits, dtype, base + tok)) + log(s)", "log(s)",
     [lambda r: t_sc.test_two_valued_row_closed_form(r, 1000, 8.0)]),
    ("wrong_sign_of_token_term", "(m - logit_at(logits, dtype, base + tok)) + log(s)",
     "(logit_at(logits, dtype, base + tok) - m) + log(s)", [lambda r: t_sc.test_two_valued_row_closed_form(r, 1000, 8.0)]),
    ("no_max_subtraction_in_result", "(m - logit_at(logits, dtype, base + tok)) + log(s)",
     "(0.0 - logit_at(logits, dtype, base + tok)) + log(s)", [lambda r: t_sc.test_uniform_row_gives_log_V(r, 1000, 17.5)]),
    ("row_stride_is_vocab_not_ld", "const int64_t base = r * ld;", "const int64_t base = r * vocab;",
     [t_sc.test_shift_invariance_and_padding]),
    ("token_of_previous_row", "const int32_t tok = token_ids[r];", "const int32_t tok = token_ids[r > 0 ? r - 1 : 0];",
     [t_sc.test_token_id_selects_the_column_not_the_row]),
    ("decay_hits_new_scores_too", "if (i < n_held) {", "if (i < n_cand) {",
     [t_se.test_decay_is_one_binary32_multiply_on_held_only]),
    ("no_decay_under_budget", "volatile float prod = E_in[i] * eta;",
     "volatile float prod = n_cand <= budget ? E_in[i] : E_in[i] * eta;",
     [t_se.test_at_or_under_budget_keeps_everything_but_still_decays]),
    ("ties_to_higher_slot", "return (a->slot > b->slot) - (a->slot < b->slot);",
     "return (a->slot < b->slot) - (a->slot > b->slot);", [t_se.test_all_ties_take_the_lowest_middle_slots]),
    ("lowest_scores_kept", "if (c != 0) return -c;", "if (c != 0) return c;",
     [t_se.test_worked_example_of_in_cache_positions]),
    ("sink_set_has_n_sink_plus_one", "for (int64_t i = 0; i < mid_lo; ++i) keep[i] = 1;",
     "for (int64_t i = 0; i <= mid_lo; ++i) keep[i] = 1;", [t_se.test_worked_example_of_in_cache_positions]),
    ("topk_over_whole_cache", "const int64_t mid_hi = n_cand - policy->n_recent;\n            for",
     "const int64_t mid_hi = n_cand;\n            for", [t_se.test_worked_example_of_in_cache_positions]),
    ("recent_window_off_by_one", "for (int64_t i = mid_hi; i < n_cand; ++i) keep[i] = 1;",
     "for (int64_t i = mid_hi + 1; i < n_cand; ++i) keep[i] = 1;", [t_se.test_k_zero_is_streamllm]),
    # ("evict at n_cand == budget" is not a mistake: with every middle slot inside the top k the
    # eviction branch keeps all slots too, so that variant computes the same function.)
    ("scores_out_not_decayed", "E_out[j] = E[i];", "E_out[j] = E_in[i];",
     [t_se.test_decay_applied_once_per_turn_sentinel]),
    ("gather_ignores_head", "+ h * S->stride_head);", "+ 0 * h * S->stride_head);",
     [t_cs.test_gather_equals_numpy_indexing_on_tagged_payload]),
    ("gather_uses_dst_slot_stride_for_src", "(size_t)((int64_t)i * S->stride_pos), row_bytes);",
     "(size_t)((int64_t)i * D->stride_pos), row_bytes);", [t_cs.test_gather_through_strided_source]),
    ("values_gathered_from_keys", "gather_one((const char*)v_src, src,", "gather_one((const char*)k_src, src,",
     [t_cs.test_gather_equals_numpy_indexing_on_tagged_payload]),
    ("lmhead_weight_read_transposed", "acc += h[k] * logit_at(weight, dtype, (int64_t)v * ld_w + k);",
     "acc += h[k] * logit_at(weight, dtype, (int64_t)k * ld_w + v);", [t_lm.test_brute_force_loops_on_a_tiny_case]),
    ("lmhead_hidden_row_stride_is_d_model", "h[k] = logit_at(hidden, dtype, r * ld_h + k);",
     "h[k] = logit_at(hidden, dtype, r * d_model + k);", [t_lm.test_leading_dimensions_skip_the_padding]),
    ("lmhead_dropped_token_term", "(float)((m - z[tok]) + log(s));", "(float)(log(s));",
     [lambda r: t_lm.test_two_valued_closed_form(r, 8.0)]),
    ("lmhead_hidden_of_row_zero", "h[k] = logit_at(hidden, dtype, r * ld_h + k);",
     "h[k] = logit_at(hidden, dtype, 0 * ld_h + k);", [lambda r: t_lm.test_matches_float64_library_matmul_and_logsumexp(r, "bf16")]),
    ("step_compacts_even_under_budget_wrong_count", "(int32_t)budget);", "(int32_t)budget - 1);",
     [t_cs.test_step_is_score_then_decay_select_then_gather]),
    # the baseline policies (Sec. 4.1) and their generator
    ("philox_nine_rounds", "for (int round = 0; round < 10; ++round) {", "for (int round = 0; round < 9; ++round) {",
     [t_bl.test_philox_known_answers]),
    ("philox_multipliers_swapped", "const uint64_t p0 = (uint64_t)0xD2511F53u * c0;\n        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;",
     "const uint64_t p0 = (uint64_t)0xCD9E8D57u * c0;\n        const uint64_t p1 = (uint64_t)0xD2511F53u * c2;",
     [t_bl.test_philox_known_answers]),
    ("philox_key_schedule_words_swapped", "k0 += 0x9E3779B9u;\n        k1 += 0xBB67AE85u;",
     "k0 += 0xBB67AE85u;\n        k1 += 0x9E3779B9u;", [t_bl.test_philox_known_answers]),
    ("philox_high_halves_not_crossed", "const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;",
     "const uint32_t n0 = (uint32_t)(p0 >> 32) ^ c1 ^ k0;", [t_bl.test_philox_known_answers]),
    ("interval_comb_anchored_at_oldest_slot", "keep[mid_hi - 1 - j * interval] = 1;", "keep[mid_lo + j * interval] = 1;",
     [t_bl.test_interval_comb_by_hand]),
    ("interval_rounded_up", "int64_t interval = M / k;", "int64_t interval = (M + k - 1) / k;",
     [t_bl.test_interval_comb_by_hand]),
    ("random_keeps_smallest_draws", "if (a->key != b->key) return a->key > b->key ? -1 : 1;",
     "if (a->key != b->key) return a->key > b->key ? 1 : -1;", [t_bl.test_random_subset_follows_the_published_generator]),
    ("random_ignores_the_stream", "(uint32_t)(mid_lo + i), (uint32_t)s, (uint32_t)turn,", "(uint32_t)(mid_lo + i), 0u, (uint32_t)turn,",
     [t_bl.test_random_subset_properties, t_bl.test_random_subset_follows_the_published_generator]),
    ("random_drops_the_turns_high_word", "(uint32_t)turn, (uint32_t)(turn >> 32)};", "(uint32_t)turn, 0u};",
     [t_bl.test_random_subset_properties]),
    ("random_counter_is_middle_relative", "const uint32_t ctr[4] = {(uint32_t)(mid_lo + i),", "const uint32_t ctr[4] = {(uint32_t)(i),",
     [t_bl.test_random_subset_follows_the_published_generator]),
    ("stream_policy_keeps_topk_slots_too", "const int64_t k = kind == 0 ? 0 : policy->n_topk;", "const int64_t k = policy->n_topk;",
     [t_bl.test_stream_policy_is_sink_plus_recent]),
]


def _load_ref_with(lib_path, tag):
    spec = importlib.util.spec_from_file_location(f"oracle.ref_{tag}", os.path.join(ROOT, "oracle", "ref.py"))
    mod = importlib.util.module_from_spec(spec)
    mod.__package__ = "oracle"
    sys.modules[spec.name] = mod
    spec.loader.exec_module(mod)
    mod._lib = mod.load(lib_path)
    return mod


@pytest.mark.parametrize("name,old,new,pins", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_reject_planted_mistake(tmp_path, name, old, new, pins):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found in the oracle source"
    (tmp_path / "sirllm_ref.c").write_text(text.replace(old, new, 1))
    shutil.copy(os.path.join(ROOT, "oracle", "sirllm_ref.h"), tmp_path / "sirllm_ref.h")
    so = str(tmp_path / f"libmut_{name}.so")
    subprocess.run(["gcc", "-std=c11", "-O1", "-fPIC", "-shared", "-fopenmp", "-w", "-o", so,
                    str(tmp_path / "sirllm_ref.c"), "-lm"], check=True)
    mref = _load_ref_with(so, name)
    caught = 0
    for pin in pins:
        try:
            pin(mref)
        except (AssertionError, ValueError):
            caught += 1
    assert caught == len(pins), f"mutant {name} slipped through"
