"""The pins must notice a plausible mistake anywhere in the oracle.

Each case plants one mistake in a copy of oracle/nd_oracle.c (a dropped term, a
wrong sign or index, a swapped operand), builds it on the CPU and runs the pin
tests against that build in a subprocess: at least one pin has to fail.  The
unmodified source must pass the same command.
"""
import os
import subprocess
import sys

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "nd_oracle.c")
PINS = ["tests/test_oracle_primitives.py", "tests/test_oracle_walks.py", "tests/test_oracle_khop_layer.py",
        "tests/test_oracle_edges.py"]

MUTANTS = {
    "philox_multipliers_swapped": ("(uint64_t)0xD2511F53u * c0", "(uint64_t)0xD2511F53u * c2"),
    "philox_key_word": ("(uint32_t)(p1 >> 32) ^ c1 ^ k0", "(uint32_t)(p1 >> 32) ^ c1 ^ k1"),
    "philox_nine_rounds": ("round < 10", "round < 9"),
    "uniform_index_shift": ("return (uint32_t)(((uint64_t)r * d) >> 32);", "return (uint32_t)(((uint64_t)r * d) >> 31) % d;"),
    "weighted_boundary": ("if (g->cumq[lo + j] > x) return j;", "if (g->cumq[lo + j] >= x) return j;"),
    "weight_rounding": ("floor((double)w[e] * 65536.0 + 0.5)", "floor((double)w[e] * 65536.0)"),
    "walk_does_not_advance": ("            out[(int64_t)i * S + s] = next;\n            v = next;\n        }\n    }\n    return 0;\n}\n\n/* ------------------------------------------------------------------------ */\n/* Personalised",
                              "            out[(int64_t)i * S + s] = next;\n        }\n    }\n    return 0;\n}\n\n/* ------------------------------------------------------------------------ */\n/* Personalised"),
    "ppr_coin_inverted": ("if ((uint64_t)r[3] >= thr) {", "if ((uint64_t)r[3] < thr) {"),
    "ppr_coin_from_the_word_that_picks_the_neighbour": ("if ((uint64_t)r[3] >= thr) {", "if ((uint64_t)r[0] >= thr) {"),
    "ppr_sample_id_base_ignored": ("draw4(seed, (uint32_t)(sample_id_base + (uint64_t)s), 0u, (uint32_t)i, 0u, r);\n                if ((uint64_t)r[3] >= thr) {",
                                   "draw4(seed, (uint32_t)s, 0u, (uint32_t)i, 0u, r);\n                if ((uint64_t)r[3] >= thr) {"),
    "n2v_sample_id_base_ignored": ("const uint32_t sid = (uint32_t)(sample_id_base + (uint64_t)s);\n        int32_t t = NDO_NULL;",
                                   "const uint32_t sid = (uint32_t)s;\n        int32_t t = NDO_NULL;"),
    "unique_refill_sample_id_base_ignored": ("draw4(seed, (uint32_t)(sample_id_base + (uint64_t)s), (uint32_t)j, (uint32_t)i,\n                          (uint32_t)r, rn);",
                                             "draw4(seed, (uint32_t)(r == 0 ? sample_id_base + (uint64_t)s : (uint64_t)s), (uint32_t)j, (uint32_t)i,\n                          (uint32_t)r, rn);"),
    "layer_step_dropped_from_the_counter": ("draw4(seed, (uint32_t)(sample_id_base + (uint64_t)b), (uint32_t)j, (uint32_t)i, 0u, r);\n                    const uint64_t x = ndo_mulhi64(((uint64_t)r[0] << 32) | r[1], total);\n                    uint64_t before = 0; /* mass of the lists in front of the current one */",
                                            "draw4(seed, (uint32_t)(sample_id_base + (uint64_t)b), (uint32_t)j, 0u, 0u, r);\n                    const uint64_t x = ndo_mulhi64(((uint64_t)r[0] << 32) | r[1], total);\n                    uint64_t before = 0; /* mass of the lists in front of the current one */"),
    "weighted_layer_step_dropped_from_the_counter": ("draw4(seed, (uint32_t)(sample_id_base + (uint64_t)b), (uint32_t)j, (uint32_t)i, 0u, r);\n                    const uint64_t x = ndo_mulhi64(((uint64_t)r[0] << 32) | r[1], total);\n                    uint64_t before = 0; /* weight of the lists in front of the current one */",
                                                     "draw4(seed, (uint32_t)(sample_id_base + (uint64_t)b), (uint32_t)j, 0u, 0u, r);\n                    const uint64_t x = ndo_mulhi64(((uint64_t)r[0] << 32) | r[1], total);\n                    uint64_t before = 0; /* weight of the lists in front of the current one */"),
    "n2v_common_and_far_swapped": ("else if (has_edge(g, t, u)) bias = b_com;\n    else bias = b_far;",
                                   "else if (has_edge(g, t, u)) bias = b_far;\n    else bias = b_com;"),
    "n2v_return_case_dropped": ("else if (u == t) bias = b_ret;", "else if (0) bias = b_ret;"),
    "n2v_envelope_not_max": ("(has_t ? b_max : NDO_ONE_Q16)", "(has_t ? b_ret : NDO_ONE_Q16)"),
    "n2v_previous_transit_stale": ("            t = v;\n            v = next;", "            v = next;"),
    "khop_parent_index": ("parent = prev[s * W_prev + j / m];", "parent = prev[s * W_prev + j % W_prev];"),
    "khop_counter_slot": ("(uint32_t)j, (uint32_t)i, 0u, r);\n                    next = g->col[g->off[parent]",
                          "(uint32_t)(j / m), (uint32_t)i, 0u, r);\n                    next = g->col[g->off[parent]"),
    "multirw_pick_word": ("ndo_uniform_index(r[2], (uint32_t)R)", "ndo_uniform_index(r[1], (uint32_t)R)"),
    "multirw_root_not_replaced": ("                cur[pick] = next;\n", ""),
    "unique_checks_lower_slots_only": ("for (int64_t q = 0; q < W && !taken; ++q)", "for (int64_t q = 0; q < j && !taken; ++q)"),
    "unique_refill_repeats_attempt_zero": ("(uint32_t)r, rn);", "0u, rn);"),
    "edges_repeated_vertex_counted_once": ("for (int32_t kk = k; kk < n_list && list[kk].v == u; ++kk) {",
                                           "for (int32_t kk = k; kk < n_list && kk < k + 1 && list[kk].v == u; ++kk) {"),
    "edges_slot_order_not_by_vertex": ("if (x->v != y->v) return x->v < y->v ? -1 : 1;\n    return x->j < y->j",
                                       "if (x->v != y->v) return x->v > y->v ? -1 : 1;\n    return x->j < y->j"),
    "edges_ties_in_falling_slot_order": ("return x->j < y->j ? -1 : (x->j > y->j);", "return x->j > y->j ? -1 : (x->j < y->j);"),
    "edges_row_pointer_off_by_one_row": ("row_ptr[b * n_prev + t] = n_edges;\n            const int32_t tv",
                                         "row_ptr[b * n_prev + t] = n_edges + (t > 0);\n            const int32_t tv"),
    "edges_first_samples_list_reused": ("const int32_t v = sampled[b * m + j];\n            if (v == NDO_NULL) continue;",
                                        "const int32_t v = sampled[j];\n            if (v == NDO_NULL) continue;"),
    "weighted_layer_lists_in_front_forgotten": ("if (g->cumq[e] > x - before) { next = g->col[e]; break; }",
                                                "if (g->cumq[e] > x) { next = g->col[e]; break; }"),
    "weighted_layer_boundary": ("if (g->cumq[e] > x - before) { next = g->col[e]; break; }",
                                "if (g->cumq[e] >= x - before) { next = g->col[e]; break; }"),
    "weighted_layer_total_misses_the_last_entry": ("total += g->cumq[g->off[v + 1] - 1];",
                                                   "total += g->off[v + 1] - 2 >= g->off[v] ? g->cumq[g->off[v + 1] - 2] : g->cumq[g->off[v + 1] - 1];"),
    "layer_weight_not_squared": ("total += d * ((((uint64_t)1) << 48) / (d * d));", "total += d * ((((uint64_t)1) << 48) / d);"),
    "layer_index_ignores_lists_in_front": ("(int64_t)((x - before) / c)", "(int64_t)((x / c) % d)"),
    "layer_total_drops_first_transit": ("for (int64_t t = 0; t < n_prev; ++t) {\n                const int32_t v = transits[t];\n                if (!valid_vertex(g, v)) continue;\n                const uint64_t d = (uint64_t)degree(g, v);\n                if (d == 0) continue;\n                if (d >= (1u << 24)) return -4;",
                                        "for (int64_t t = 1; t < n_prev; ++t) {\n                const int32_t v = transits[t];\n                if (!valid_vertex(g, v)) continue;\n                const uint64_t d = (uint64_t)degree(g, v);\n                if (d == 0) continue;\n                if (d >= (1u << 24)) return -4;"),
}


def _run_pins(lib):
    env = dict(os.environ, ND_ORACLE_LIB=lib)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PINS]
    return subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True)


def test_unmodified_oracle_passes_the_pins(tmp_path):
    lib = str(tmp_path / "clean.so")
    oracle.compile_oracle(SRC, lib)
    r = _run_pins(lib)
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new, 1))
    lib = str(tmp_path / "mutant.so")
    oracle.compile_oracle(str(src), lib)
    r = _run_pins(lib)
    assert r.returncode != 0, f"no pin noticed the planted mistake '{name}'"
