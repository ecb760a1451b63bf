"""The pins must bite: plant one plausible mistake at a time in a private copy of the
oracle's source (CPU only), swap it in, and check that a named pin fails.

The mutated copy is built by replacing one snippet of the oracle's text; each snippet
must occur exactly once, so a change to the oracle that makes a mutant meaningless
breaks this file loudly instead of silently weakening it.
"""
import inspect
import types

import pytest

from oracle import lukv_oracle as O
from tests import test_oracle_allocate as TA
from tests import test_oracle_score as TS
from tests import test_oracle_topk_alloc as TK

PUBLIC = ["window_attention_sum", "window_lse", "max_pool_1d", "score", "concave_hull", "marginal_gains",
          "_gain_of_unit", "_slope", "allocate", "select", "compact", "offsets_of", "profile_build",
          "budgets_from_profile", "decode_attention", "utility_curve", "allocate_topk"]

MUTANTS = {
    # name: (snippet, replacement, pin that must fail)
    "dropped_group_mean": ("out[c] = acc / G", "out[c] = acc",
                           lambda: TS.test_identical_keys_closed_form_and_group_mean()),
    "non_causal_window": ("visible = j <= t ", "visible = j <= L ",
                          lambda: TS.test_handworked_unpooled_is_causal()),
    "strictly_causal_window": ("visible = j <= t ", "visible = j < t ",
                               lambda: TS.test_identical_keys_closed_form_and_group_mean()),
    "mean_over_window": ("acc += p.sum(axis=0)", "acc += p.mean(axis=0)",
                         lambda: TS.test_total_mass_is_window_size()),
    "missing_scale": ("scale = 1.0 / math.sqrt(d)\n    out = np.zeros((H_kv, L)", "scale = 1.0\n    out = np.zeros((H_kv, L)",
                      lambda: TS.test_brute_force_definition()),
    "softmax_over_queries": ("p = e / e.sum(axis=1, keepdims=True)",
                             "p = e / e.sum(axis=0, keepdims=True)",
                             lambda: TS.test_total_mass_is_window_size()),
    "pool_window_shifted": ("out = np.maximum(out, padded[..., t:t + n])",
                            "out = np.maximum(out, padded[..., t + 1:t + 1 + n] if t + 1 + n <= "
                            "padded.shape[-1] else out)",
                            lambda: TS.test_pool_properties_and_library_cross_check()),
    "pool_over_window_too": ("s[:, :P] = max_pool_1d(r[:, :P], pool_kernel)",
                             "s[:, :P] = max_pool_1d(r, pool_kernel)[:, :P]",
                             lambda: TS.test_handworked_pool_stays_inside_prefix()),
    "lse_added_not_subtracted": ("p = np.exp(s - np.asarray(lse[c * G + g]", "p = np.exp(s + np.asarray(lse[c * G + g]",
                                 lambda: TS.test_handworked_lse_variant()),
    "lse_of_wrong_head": ("p = np.exp(s - np.asarray(lse[c * G + g]", "p = np.exp(s - np.asarray(lse[c + g]",
                          lambda: TS.test_lse_variant_equals_recomputed_normaliser()),
    "lse_not_causal": ("row = s[i, :L - w + i + 1]", "row = s[i, :]",
                       lambda: TS.test_handworked_lse_variant()),
    "profile_keeps_instead_of_evicts": ("acc = acc + (1.0 - b.astype(np.float64) / float(L))",
                                        "acc = acc + (b.astype(np.float64) / float(L))",
                                        lambda: TA.test_handworked_profile_and_lookup()),
    "profile_budget_from_rho_not_one_minus_rho": ("B = int(math.floor((1.0 - float(r)) * float(L) * float(NH)))",
                                                  "B = int(math.floor(float(r) * float(L) * float(NH)))",
                                                  lambda: TA.test_handworked_profile_and_lookup()),
    "lookup_rounds_instead_of_floor": ("b = np.floor((1.0 - r) * float(L)).astype(np.int64)",
                                       "b = np.rint((1.0 - r) * float(L)).astype(np.int64)",
                                       lambda: TA.test_handworked_profile_and_lookup()),
    "lookup_no_interpolation": ("r = lo + t * (hi - lo)", "r = lo",
                                lambda: TA.test_handworked_profile_and_lookup()),
    "decode_softmax_over_queries": ("p = p / p.sum(axis=1, keepdims=True)\n    return p @ v_rows",
                                    "p = p / p.sum(axis=0, keepdims=True)\n    return p @ v_rows",
                                    lambda: TS.test_decode_attention_library_cross_check()),
    "decode_missing_scale": ("scale = 1.0 / math.sqrt(d)\n    if k_rows.shape[0] == 0:", "scale = 1.0\n    if k_rows.shape[0] == 0:",
                             lambda: TS.test_decode_attention_library_cross_check()),
    "decode_values_for_keys": ("return p @ v_rows", "return p @ k_rows",
                               lambda: TS.test_decode_attention_handworked_and_special_cases()),
    "curve_ranks_ascending": ('order = np.argsort(-np.asarray(scores, dtype=np.float64), kind="stable")\n    u =',
                              'order = np.argsort(np.asarray(scores, dtype=np.float64), kind="stable")\n    u =',
                              lambda: TA.test_handworked_utility_curve_and_properties()),
    "curve_sums_unranked": ("np.cumsum(np.asarray(importance, dtype=np.float64)[order])",
                            "np.cumsum(np.asarray(importance, dtype=np.float64))",
                            lambda: TA.test_handworked_utility_curve_and_properties()),
    "sink_not_forced": ("s[:, :min(n_sink, L)] = np.inf", "pass",
                        lambda: TS.test_brute_force_definition()),
    "hull_keeps_collinear": ("<= _slope(knots, U, ends[-2], ends[-1]):", "< _slope(knots, U, ends[-2], ends[-1]):",
                             lambda: TA.test_collinear_knots_are_not_vertices()),
    "hull_pools_only_once": ("while len(ends) >= 3 and _slope(", "if len(ends) >= 3 and _slope(",
                             lambda: TA.test_pooling_cascades_and_uses_the_pooled_blocks_own_chord()),
    "hull_compares_last_interval_not_pooled_block": ("<= _slope(knots, U, ends[-2], ends[-1]):",
                                                     "<= _slope(knots, U, g - 1, g):",
                                                     lambda: TA.test_pooling_cascades_and_uses_the_pooled_blocks_own_chord()),
    "hull_lower_instead_of_upper": ("<= _slope(knots, U, ends[-2], ends[-1]):", ">= _slope(knots, U, ends[-2], ends[-1]):",
                                    lambda: TA.test_handworked_hull_and_gains()),
    "gain_run_over_rise": ("return float((np.float64(U[b]) - np.float64(U[a])) / np.float64(int(knots[b]) - int(knots[a])))",
                           "return float(np.float64(int(knots[b]) - int(knots[a])) / (np.float64(U[b]) - np.float64(U[a]) + 1e-30))",
                           lambda: TA.test_handworked_hull_and_gains()),
    "segment_owner_off_by_one": ("if lo < u <= hi:", "if lo <= u < hi:",
                                 lambda: TA.test_handworked_hull_and_gains()),
    "head_tie_highest_first": ("h = int(np.argmax(nxt)) ", "h = int(len(nxt) - 1 - np.argmax(nxt[::-1])) ",
                               lambda: TA.test_handworked_budgets_all_B()),
    "min_retention_ignored": ("budgets = np.array([int(x) for x in b_min], dtype=np.int64)",
                              "budgets = np.array([0 for x in b_min], dtype=np.int64)",
                              lambda: TA.test_handworked_budgets_all_B()),
    "topk_ties_unstable_order": ('order = np.argsort(-s.astype(np.float64), kind="stable")',
                                 'order = np.argsort(-s.astype(np.float64)[::-1], kind="stable")[::1]; '
                                 'order = len(s) - 1 - order',
                                 lambda: TS.test_handworked_topk_lowest_index_ties()),
    "topk_smallest": ('order = np.argsort(-s.astype(np.float64), kind="stable")',
                      'order = np.argsort(s.astype(np.float64), kind="stable")',
                      lambda: TA.test_select_brute_force_with_ties(0)),
    "global_topk_takes_smallest": ("order = np.lexsort((pos, head, -val))", "order = np.lexsort((pos, head, val))",
                                   lambda: TK.test_handworked_global_topk()),
    "global_topk_ties_to_highest_head": ("order = np.lexsort((pos, head, -val))",
                                         "order = np.lexsort((pos, -head, -val))",
                                         lambda: TK.test_ties_go_to_the_lowest_head_then_the_lowest_position()),
    "global_topk_floor_counted_twice": ("outside[select(np.asarray(s), floor)] = False", "pass",
                                        lambda: TK.test_handworked_global_topk()),
    "global_topk_floor_not_deducted": ("taken = order[:B_total - H * floor]", "taken = order[:B_total]",
                                       lambda: TK.test_handworked_global_topk()),
    "global_topk_floor_guards_worst_positions": ("outside[select(np.asarray(s), floor)] = False",
                                                 "outside[select(-np.asarray(s), floor)] = False",
                                                 lambda: TK.test_equals_exhaustive_search_on_tiny_inputs(0)),
    "global_topk_accepts_too_large_B": ("or B_total < H * floor or B_total > sum(lens):",
                                        "or B_total < H * floor:",
                                        lambda: TK.test_infeasible_cases()),
}


def _mutated_module(snippet, replacement):
    src = inspect.getsource(O)
    assert src.count(snippet) == 1, "mutation target must occur exactly once: %r" % snippet
    mod = types.ModuleType("lukv_oracle_mutant")
    exec(compile(src.replace(snippet, replacement), "lukv_oracle_mutant", "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name, monkeypatch):
    snippet, replacement, pin = MUTANTS[name]
    mutant = _mutated_module(snippet, replacement)
    for fn in PUBLIC:
        monkeypatch.setattr(O, fn, getattr(mutant, fn))
    with pytest.raises(AssertionError):
        pin()


def test_unmutated_copy_passes_the_same_pins(monkeypatch):
    """Control: the swap mechanism itself does not make pins fail."""
    clean = _mutated_module("out[c] = acc / G", "out[c] = acc / G ")
    for fn in PUBLIC:
        monkeypatch.setattr(O, fn, getattr(clean, fn))
    for _, _, pin in MUTANTS.values():
        pin()
