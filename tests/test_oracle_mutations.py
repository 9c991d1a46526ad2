"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's source (a wrong
sign, a dropped term, a missing step), builds it, and runs the pin tests that should notice: they
must fail.  Everything here happens on the CPU, on copies; the oracle itself is not touched."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ggnn_ref.c")

MUTATIONS = [
    # (name, text in ggnn_ref.c, replacement, pin tests expected to fail)
    ("difference_becomes_sum", "float t = q[j] - x;", "float t = q[j] + x;", "distance_l2_exact"),
    ("all_chunks_on_one_accumulator", "int l = c % lanes;", "int l = 0;", "summation_tree"),
    ("square_root_dropped", "return sqrtf(tree_sum(q, row, D, dtype, lanes, 0));", "return tree_sum(q, row, D, dtype, lanes, 0);",
     "distance_l2_exact"),
    ("cosine_sign", "return fmaxf(0.0f, 1.0f - dot);", "return fmaxf(0.0f, 1.0f + dot);", "distance_cosine"),
    ("order_by_distance_reversed", "return a.d < b.d || (a.d == b.d && a.id < b.id);",
     "return a.d > b.d || (a.d == b.d && a.id < b.id);", "bruteforce_matches_float64"),
    ("geometry_takes_the_worse_factor", "if (best_g < 0 || err < best_err) {", "if (best_g < 0 || err > best_err) {",
     "geometry_matches_paper"),
    ("inverse_partition_runs_rounds_forward", "for (int r = 3; r >= 0; r--) {", "for (int r = 0; r < 4; r++) {",
     "partition_is_a_bijection"),
    ("known_points_not_removed_from_proposals", "    if (cache_known(c, p)) continue;\n", "", "unbounded_best"),
    ("push_forgets_prioq", "  sorted_insert(c->pq, &c->np, c->P, e);\n", "", "unbounded_best"),
    ("pop_ignores_the_criterion", "  if (!cache_crit(c, c->pq[0].d)) return -1;\n", "", "classical_best_first"),
    ("slack_dropped_from_threshold", "  return dk + xi;", "  return dk;", "slack_monotone"),
    ("transform_keeps_old_ids", "  for (int i = 0; i < c->nb; i++) c->best[i].id = table[c->best[i].id];\n", "",
     "unbounded_best"),
    ("merge_admits_the_point_itself", "        if (base_of(g, l_m, mem[i]) == zb) continue;\n", "", "merge_on_own_layer"),
    ("mean_not_divided", "g->stats[0] = (float)(sum / (double)g->N);", "g->stats[0] = (float)sum;", "merge_on_own_layer"),
    ("reservoir_key_multiplies", "key[i] = (w > 0.0) ? log(u) / w : -INFINITY;", "key[i] = (w > 0.0) ? log(u) * w : -INFINITY;",
     "select_ranks"),
    ("unequal_shares", "int share = (int)(((int64_t)(j + 1) * g->s) / g->g - ((int64_t)j * g->s) / g->g);",
     "int share = (j == 0) ? g->s : 0;", "select_takes_equal_shares"),
    ("inverse_links_take_one_slot_too_many", "      keep = (valid < K - nl) ? valid : K - nl;",
     "      keep = (valid < K - nl - 1) ? valid : K - nl - 1;", "sym_adds_back_links"),
    ("midpoint_constraint_ignored_in_radius", "      c.radius = ggnn_ref_distance(q, row_ptr(g, xb), g->D, row_dtype(g), g->metric, g->lanes);",
     "      c.radius = 0.0f;", "sym_adds_back_links"),
    ("shard_offsets_dropped", "        e.id = id + offsets[s];", "        e.id = id;", "shard_merge"),
]


@pytest.mark.parametrize("name,old,new,pins", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch_planted_mistake(tmp_path, name, old, new, pins):
    src = open(SRC).read()
    assert src.count(old) == 1, "mutation site not unique: %s" % name
    mutated = tmp_path / "ggnn_ref.c"
    mutated.write_text(src.replace(old, new))
    (tmp_path / "ggnn_ref.h").write_text(open(os.path.join(ROOT, "oracle", "ggnn_ref.h")).read())
    lib = tmp_path / "libggnn_ref_mutant.so"
    subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", str(mutated), "-o", str(lib), "-lm"],
                   check=True, capture_output=True)
    env = dict(os.environ, GGNN_REF_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-k", pins, "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 1, "the pins did not notice '%s':\n%s" % (name, r.stdout[-1500:])
    assert "failed" in r.stdout
