"""Are the pins sharp?  Each case plants one plausible mistake in a copy of the oracle's C source
(a wrong index, a dropped term, a wrong rounding, a transposed role), builds that copy, points the
oracle package at it and requires that the named pins fail.  A pin that still passes on a broken
oracle would not be pinning anything.  CPU only; the real oracle is never modified."""
import os
import subprocess
import sys

import pytest

# (name, text in oracle/hmo.c, replacement, pins expected to notice: "module:function" or
#  ("module:function", kwargs) for parametrised ones).  Every planted mistake keeps all memory
# accesses in bounds.
MUTATIONS = [
    ("gpu level deduplicates per node",
     "return level == HMO_LEVEL_NODE ? rank / ranks_per_node : rank;",
     "return level != HMO_LEVEL_NONE ? rank / ranks_per_node : rank;",
     ["test_oracle_plan_pins:test_random_small_tables_match_set_definition"]),
    ("first-occurrence test looks at the previous slot only",
     "for (int32_t k1 = 0; k1 < k; ++k1)\n                    if (dest[(size_t)t * K + k1] == dest[s]) keep = 0;",
     "for (int32_t k1 = (k > 0 ? k - 1 : 0); k1 < k; ++k1)\n                    if (dest[(size_t)t * K + k1] == dest[s]) keep = 0;",
     ["test_oracle_plan_pins:test_random_small_tables_match_set_definition"]),
    ("row weight forgets the later slots of a row",
     "else            { row_weight[row] = row_weight[row] + topk_weights[s]; }",
     "else            { }",
     [("test_oracle_plan_pins:test_level_invariants", dict(name="qwen3"))]),
    ("combine pairs a row with the next slot's weight",
     "acc += (double)topk_weights[t * K + k] * bf16_to_f64(y[row * H + j]);",
     "acc += (double)topk_weights[t * K + (k + 1) % K] * bf16_to_f64(y[row * H + j]);",
     ["test_oracle_data_pins:test_combine_exact_rational_small"]),
    ("combine accumulates in binary32",
     "            double acc = 0.0;\n            for (int32_t k = 0; k < K; ++k) {\n                const int64_t row = slot_row[t * K + k];\n"
     "                if (row < 0) continue;\n                if (row >= y_rows) return HMO_ERR_ARG;\n"
     "                acc += (double)topk_weights[t * K + k] * bf16_to_f64(y[row * H + j]);",
     "            float acc = 0.0;\n            for (int32_t k = 0; k < K; ++k) {\n                const int64_t row = slot_row[t * K + k];\n"
     "                if (row < 0) continue;\n                if (row >= y_rows) return HMO_ERR_ARG;\n"
     "                acc += (double)topk_weights[t * K + k] * bf16_to_f64(y[row * H + j]);",
     ["test_oracle_data_pins:test_combine_accumulates_beyond_binary32"]),
    ("bf16 rounding truncates",
     "const double q = nearbyint(ldexp(v, -ulp_exp));", "const double q = trunc(ldexp(v, -ulp_exp));",
     ["test_oracle_data_pins:test_bf16_rounding_against_exact_rationals"]),
    ("bf16 rounding breaks ties away from zero",
     "const double q = nearbyint(ldexp(v, -ulp_exp));", "const double q = round(ldexp(v, -ulp_exp));",
     ["test_oracle_data_pins:test_bf16_rounding_against_exact_rationals"]),
    ("bf16 subnormal spacing off by one binade",
     "if (ulp_exp < -133) ulp_exp = -133;", "if (ulp_exp < -134) ulp_exp = -134;",
     ["test_oracle_data_pins:test_bf16_rounding_against_exact_rationals"]),
    ("transpose takes the weight of another row",
     "volatile float p = row_weight[row] * gout[(int64_t)t * H + j];",
     "volatile float p = row_weight[t % n_rows] * gout[(int64_t)t * H + j];",
     [("test_oracle_data_pins:test_transpose_is_adjoint_and_one_multiply", dict(level=1))]),
    ("bf16 transpose rounds twice (binary32, then bf16)",
     "gy[row * H + j] = f64_to_bf16_rne((double)row_weight[row] * bf16_to_f64(gout[(int64_t)t * H + j]));",
     "gy[row * H + j] = f64_to_bf16_rne((double)(float)((double)row_weight[row] * bf16_to_f64(gout[(int64_t)t * H + j])));",
     ["test_oracle_data_pins:test_transpose_bf16_exact_products_and_double_rounding_trap"]),
    ("load_rank counts slots, not tokens",
     "in_rank[rank] = 1;", "in_rank[rank] += 1;",
     [("test_oracle_plan_pins:test_level_invariants", dict(name="qwen3"))]),
    ("node mask built from the rank",
     "nm |= (uint32_t)1 << (rank / ranks_per_node);", "nm |= (uint32_t)1 << (rank % 32);",
     ["test_oracle_plan_pins:test_random_small_tables_match_set_definition",
      ("test_oracle_plan_pins:test_level_invariants", dict(name="qwen3"))]),
    ("fp32 combine accumulates in binary32",
     "acc += (double)topk_weights[t * K + k] * (double)y[row * H + j];",
     "acc = (float)(acc + (double)((float)topk_weights[t * K + k] * y[row * H + j]));",
     ["test_oracle_data_pins:test_combine_f32_accumulates_beyond_binary32"]),
    ("fp32 combine lets dropped slots contribute",
     "                if (row < 0) continue;\n                if (row >= y_rows) return HMO_ERR_ARG;\n"
     "                acc += (double)topk_weights[t * K + k] * (double)y[row * H + j];",
     "                if (row < 0) { acc += 1e-3; continue; }\n                if (row >= y_rows) return HMO_ERR_ARG;\n"
     "                acc += (double)topk_weights[t * K + k] * (double)y[row * H + j];",
     ["test_oracle_data_pins:test_combine_f32_is_plain_weighted_sum_and_agrees_with_bf16_combine"]),
    ("swap_apply writes one entry only",
     "    expert_to_rank[c] = g;\n", "    expert_to_rank[c] = expert_to_rank[c];\n",
     ["test_oracle_swap_pins:test_swap_apply_and_the_planner_loop"]),
    ("intra-node table divides where it should take the remainder",
     "? g % ranks_per_node : -1;", "? g / ranks_per_node : -1;",
     ["test_oracle_recv_pins:test_dest_maps_against_numpy"]),
    ("local expert indices do not ascend with the expert id",
     "dest_map[e] = (g == my_rank) ? next_local++ : -1;", "dest_map[e] = (g == my_rank) ? (E - 1 - next_local++) % 64 : -1;",
     ["test_oracle_recv_pins:test_dest_maps_against_numpy"]),
    ("hop table: child index not taken inside the parent",
     "else dest_map[e] = (g / ranks_per_child) % children_per_parent;", "else dest_map[e] = (g / ranks_per_child);",
     ["test_oracle_recv_pins:test_level_dest_map_against_numpy"]),
    ("hop table: membership tested on the child group",
     "else if (g / ranks_per_parent != my_rank / ranks_per_parent) dest_map[e] = -1;",
     "else if (g / ranks_per_child != my_rank / ranks_per_child) dest_map[e] = -1;",
     ["test_oracle_recv_pins:test_level_dest_map_against_numpy"]),
    ("normalised merge does not normalise",
     "out[i * H + j] = f64_to_bf16_rne(wsum != 0.0 ? acc / wsum : 0.0);", "out[i * H + j] = f64_to_bf16_rne(acc);",
     ["test_oracle_recv_pins:test_combine_mix_exact_rational"]),
    ("normalised merge divides by the weights of skipped slots too",
     "if (slot_row[i * K + k] >= 0) wsum += (double)weights[i * K + k];", "wsum += (double)weights[i * K + k];",
     ["test_oracle_recv_pins:test_combine_mix_exact_rational"]),
    ("time model: inter-level fan-out is U[i], not U[i]/U[i-1]",
     "const double n = (double)(U[i] / U[i - 1]) * max_count(p_inter + i * 64, U[i]) * M * v;",
     "const double n = (double)(U[i]) * max_count(p_inter + i * 64, U[i]) * M * v;",
     ["test_oracle_model_pins:test_four_dimensions_with_the_papers_parameters"]),
    ("time model: intra-level maximum over too few peers",
     "const double n = (double)(G / U[d - 1]) * max_count(p_intra + (d - 1) * 64, G) * M * v;",
     "const double n = (double)(G / U[d - 1]) * max_count(p_intra + (d - 1) * 64, U[d - 1]) * M * v;",
     ["test_oracle_model_pins:test_one_dimension_is_eq1_eq2", "test_oracle_model_pins:test_two_dimensions_by_hand"]),
    ("d*: one dimension wins only by a factor of two",
     "if (times[0] < times[arg - 1]) arg = 1;", "if (times[0] <= times[arg - 1] * 0.5) arg = 1;",
     ["test_oracle_model_pins:test_eq6_selection_rule"]),
    ("swap update: gain although the group already had an expert",
     "const int gain = in_group[gb] == 0;", "const int gain = in_group[gb] <= 1;",
     ["test_oracle_swap_pins:test_incremental_update_equals_definition"]),
    ("swap update: loss although the group keeps another expert",
     "const int loss = in_group[ga] == 1;", "const int loss = in_group[ga] >= 1;",
     ["test_oracle_swap_pins:test_incremental_update_equals_definition"]),
    ("swap update: Z not symmetric",
     "zab[gb] += gain; zba[gb] += gain;", "zab[gb] += gain;",
     ["test_oracle_swap_pins:test_incremental_update_equals_definition"]),
    ("smooth maximum: wrong root",
     "return m * pow(sum, 1.0 / gamma);", "return m * pow(sum, 1.0 / (gamma + 1.0));",
     ["test_oracle_swap_pins:test_smooth_max_and_selection"]),
    ("Q: alpha and beta exchanged",
     "q = q + (n * beta_intra + alpha_intra);", "q = q + (n * alpha_intra + beta_intra);",
     ["test_oracle_swap_pins:test_smooth_max_and_selection"]),
    ("argmin keeps the last minimiser",
     "if (br < 0 || q < best) { best = q; br = r; bc = c; }", "if (br < 0 || q <= best) { best = q; br = r; bc = c; }",
     ["test_oracle_swap_pins:test_smooth_max_and_selection"]),
]


_CHILD = r"""
import ctypes, importlib, sys
sys.path.insert(0, {tests!r}); sys.path.insert(0, {root!r})
import oracle
oracle._load()
mutant = ctypes.CDLL({so!r})
mutant.hmo_f64_to_bf16.restype = ctypes.c_uint16
mutant.hmo_f64_to_bf16.argtypes = [ctypes.c_double]
pins = {pins!r}
def run(spec):
    target, kwargs = (spec, {{}}) if isinstance(spec, str) else spec
    mod, fn = target.split(":")
    getattr(importlib.import_module(mod), fn)(oracle, **kwargs)
for spec in pins:
    run(spec)                                     # every pin passes on the real oracle ...
oracle._lib = mutant
noticed = 0
for spec in pins:
    try:
        run(spec)
    except (AssertionError, IndexError, ValueError):
        noticed += 1
sys.exit(10 if noticed else 11)                   # ... and at least one must fail on the broken one
"""


@pytest.mark.parametrize("name,old,new,pins", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(oracle, tmp_path, name, old, new, pins):
    here = os.path.dirname(os.path.abspath(__file__))
    src = open(os.path.join(os.path.dirname(oracle.__file__), "hmo.c")).read()
    assert src.count(old) >= 1, "the oracle no longer contains the text this case edits"
    c_file, so_file = tmp_path / "hmo_mutant.c", tmp_path / "libhmo_mutant.so"
    c_file.write_text(src.replace(old, new, 1))
    subprocess.check_call(["gcc", *oracle.CFLAGS, "-o", str(so_file), str(c_file), "-lm"])
    # in a child process: a broken oracle must not be able to take the test run down with it
    code = _CHILD.format(tests=here, root=os.path.dirname(here), so=str(so_file), pins=pins)
    rc = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert rc.returncode in (10, 11), "child failed outside the pins (rc %d): %s" % (rc.returncode, rc.stderr[-2000:])
    assert rc.returncode == 10, "no pin noticed: %s" % name
