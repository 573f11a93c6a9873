"""The pins must be sharp: a plausible mistake planted in a copy of the oracle's source
(on the CPU, never in the GPU code) has to make at least one pin fail."""
import os
import subprocess

import numpy as np
import pytest

import test_oracle_pins as pins
import test_oracle_reusable as reusable
import test_oracle_layers as layers
import test_oracle_orders as orders
import test_oracle_fusion as fusion

MUTATIONS = {
    "closed_lifetimes": ("return ts_a < te_b && ts_b < te_a;", "return ts_a <= te_b && ts_b <= te_a;"),
    "closed_ranges": ("return a_a < a_b + s_b && a_b < a_a + s_a;", "return a_a <= a_b + s_b && a_b <= a_a + s_a;"),
    "previous_end_not_max": ("if (spans[c].end > x) x = spans[c].end;", "x = spans[c].end;"),
    "hole_needs_extra_byte": ("if (spans[c].a >= x + s) break;", "if (spans[c].a > x + s) break;"),
    "lists_ignore_placed": ("if (placed[j]) { spans[m].a", "if (1) { spans[m].a"),
    "live_includes_release_time": ("if (t_s[i] <= t && t < t_e[i]) live += size[i];",
                                   "if (t_s[i] <= t && t <= t_e[i]) live += size[i];"),
    "sweep_drops_release": ("net[t_e[i]] -= (int64_t)size[i];", "net[t_e[i]] -= 0;"),
    "validate_skips_neighbour": ("for (uint32_t j = i + 1; j < n; ++j)\n            if (lifetimes_conflict(t_s[i], t_e[i], t_s[j], t_e[j]) &&",
                                 "for (uint32_t j = i + 2; j < n; ++j)\n            if (lifetimes_conflict(t_s[i], t_e[i], t_s[j], t_e[j]) &&"),
    "best_plan_last_of_equals": ("if (extent[p] < extent[b]) b = p;", "if (extent[p] <= extent[b]) b = p;"),
    "sort_descending": ("if (x->a != y->a) return x->a < y->a ? -1 : 1;", "if (x->a != y->a) return x->a < y->a ? 1 : -1;"),
    "window_closed": ("if (lifetimes_conflict(t_s[i], t_e[i], w_lo, w_hi)) {", "if (t_s[i] <= w_hi && w_lo <= t_e[i]) {"),
    "idle_reach_not_max": ("if (c < k && met[c].end > reach) reach = met[c].end;", "if (c < k) reach = met[c].end;"),
    "idle_pool_from_zero": ("uint64_t pool_lo = a[0], pool_hi = a[0] + size[0];", "uint64_t pool_lo = 0, pool_hi = a[0] + size[0];"),
    "idle_no_tail_interval": ("for (size_t c = 0; c <= k; ++c) {", "for (size_t c = 0; c < k; ++c) {"),
    "idle_count_capped": ("            ++found;\n            total += next - reach;", "            if (found < cap) ++found;\n            total += next - reach;"),
    "idle_needs_gap_of_two": ("if (next > reach) {", "if (next > reach + 1) {"),
    "layer_first_free_not_latest": ("l = pile[--on_pile];", "l = pile[0]; pile[0] = pile[--on_pile];"),
    "layer_needs_idle_tick": ("if (x->is_alloc != y->is_alloc) return x->is_alloc < y->is_alloc ? -1 : 1;",
                              "if (x->is_alloc != y->is_alloc) return x->is_alloc > y->is_alloc ? -1 : 1;"),
    "layer_shared_across_groups": ("uint32_t on_pile = 0;                  /* every group starts with no layer */",
                                   "static uint32_t on_pile; if (g0 == 0) on_pile = 0;"),
    "layer_end_not_updated": ("                layer_of[i] = l;\n                layer_t_e[l] = t_e[i];",
                              "                layer_of[i] = l;\n                if (l + 1 == layers) layer_t_e[l] = t_e[i];"),
    "layer_groups_ascending": ("if (x->size != y->size) return x->size > y->size ? -1 : 1;\n    return x->id < y->id ? -1 : (x->id > y->id ? 1 : 0);\n}\n\nstatic int by_time_release_first",
                               "if (x->size != y->size) return x->size > y->size ? 1 : -1;\n    return x->id < y->id ? -1 : (x->id > y->id ? 1 : 0);\n}\n\nstatic int by_time_release_first"),
    "layer_equal_starts_by_highest_number": ("    return x->id < y->id ? -1 : (x->id > y->id ? 1 : 0);\n}\n\nstatic int descending_u32",
                                             "    return x->id > y->id ? -1 : (x->id < y->id ? 1 : 0);\n}\n\nstatic int descending_u32"),
    "layer_equal_ends_opened_last_first": ("return (x < y) - (x > y);", "return (x > y) - (x < y);"),
    "orders_jitter_one_bit_short": ("<< 32) + (k >> 31); }", "<< 32) + (k >> 32); }"),
    "orders_lifetime_row_by_size_first": ("{ m[i].k0 = ~(uint64_t)(t_e[i] - t_s[i]); m[i].k1 = ~size[i]; }",
                                          "{ m[i].k1 = ~(uint64_t)(t_e[i] - t_s[i]); m[i].k0 = ~size[i]; }"),
    "orders_generator_shift": ("z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;", "z = (z ^ (z >> 28)) * 0x94D049BB133111EBull;"),
    "orders_counter_not_spread": ("(uint64_t)i * 0xD1342543DE82EF95ull + stream", "(uint64_t)i + stream"),
    "orders_classes_ascending": ("return x > y ? -1 : (x < y ? 1 : 0);", "return x > y ? 1 : (x < y ? -1 : 0);"),
    "fusion_larger_plan_by_earliest_release": ("if (a->key != b->key) return a->key > b->key ? -1 : 1;", "if (a->key != b->key) return a->key > b->key ? 1 : -1;"),
    "fusion_latest_request_first": ("if (a->key != b->key) return a->key < b->key ? -1 : 1;\n    return a->id < b->id ? -1 : (a->id > b->id ? 1 : 0);\n}\n\nint oracle_fuse_groups",
                                    "if (a->key != b->key) return a->key < b->key ? 1 : -1;\n    return a->id < b->id ? -1 : (a->id > b->id ? 1 : 0);\n}\n\nint oracle_fuse_groups"),
    "fusion_accepts_equal_product": ("*accepted_out = rf < r1 + r2 ? 1u : 0u;", "*accepted_out = rf <= r1 + r2 ? 1u : 0u;"),
    "fusion_jumps_to_the_highest_address": ("if (addr_out[k] > addr && (!have || addr_out[k] < next))", "if (addr_out[k] > addr && (!have || addr_out[k] > next))"),
    "fusion_addr_not_advanced": ("            addr += size[ks[fit].id];\n", "            addr += 0;\n"),
    "fusion_leftovers_at_the_larger_plans_top": ("        if (end > top) top = end;\n    }\n    for (uint32_t k = 0; k < ns; ++k) {\n        if (placed[k]) continue;", "        if (end > top && q < nl) top = end;\n    }\n    for (uint32_t k = 0; k < ns; ++k) {\n        if (placed[k]) continue;"),
    "extent_forgets_size": ("if (a[i] + size[i] > top) top = a[i] + size[i];\n    }\n    free(spans);\n    *extent",
                            "if (a[i] > top) top = a[i];\n    }\n    free(spans);\n    *extent"),
}


def _battery(oracle):
    for name in pins.GOLDEN:
        for method in ("allpairs", "lists"):
            pins.test_hand_worked_examples(oracle, name, method)
    pins.test_time_clique_gives_prefix_sums(oracle)
    pins.test_time_disjoint_all_at_zero(oracle)
    pins.test_equal_sizes_start_order_reaches_layer_count(oracle, 0)
    pins.test_stack_discipline_reaches_lower_bound(oracle)
    for seed in range(6):
        pins.test_all_orders_reach_exact_optimum(oracle, seed)
        pins.test_random_traces_valid_and_minimal(oracle, seed, False)
        pins.test_validate_counts_planted_conflicts(oracle, seed)
    pins.test_validate_known_single_conflict(oracle)
    pins.test_best_plan_prefers_lowest_index(oracle)
    reusable.test_hand_worked_windows(oracle)
    reusable.test_closed_forms(oracle)
    for seed in range(6):
        reusable.test_matches_byte_map(oracle, seed)
    reusable.test_lowest_fit_plans_have_no_idle_space_over_the_whole_iteration(oracle, 0)
    orders.test_splitmix64_published_outputs(oracle)
    orders.test_rows_are_permutations_and_heuristic_rows_follow_their_rules(oracle, 0)
    orders.test_matches_the_input_generator(oracle, 1)
    orders.test_random_families_have_the_intended_statistics(oracle)
    layers.test_hand_worked_example(oracle)
    layers.test_closed_forms(oracle)
    for seed in range(4):
        layers.test_random_traces_structure_and_minimum(oracle, seed)
        layers.test_layers_planned_as_requests_expand_to_a_valid_plan(oracle, seed)
    fusion.test_hand_worked_fusions(oracle)
    fusion.test_closed_forms(oracle)
    fusion.test_first_placement_is_the_earliest_request_that_fits_at_the_lowest_start_address(oracle)
    for seed in range(12):
        fusion.test_fused_plans_are_valid_and_the_accept_test_is_the_tmp_test(oracle, seed)


def test_battery_passes_on_the_real_oracle(oracle):
    _battery(oracle)


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(oracle, tmp_path, name):
    old, new = MUTATIONS[name]
    src = open(os.path.join(os.path.dirname(oracle.__file__), "stalloc_oracle.c")).read()
    assert src.count(old) >= 1, "mutation target not found in the oracle source"
    c_file = tmp_path / "mutant.c"
    so_file = tmp_path / "mutant.so"
    c_file.write_text(src.replace(old, new))
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-shared", "-fPIC", "-o", str(so_file), str(c_file)])
    with oracle.use_library(str(so_file)):
        with pytest.raises(AssertionError):
            _battery(oracle)
