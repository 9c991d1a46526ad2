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
    # ---- the stopping rule (Eq. 2 - Eq. 4), caught by the hand-worked cases
    ("slack_takes_the_larger_of_best_and_dnn", "fminf(c->best[0].d, c->dnn)", "fmaxf(c->best[0].d, c->dnn)",
     "slack_uses_the_smaller or slack_is_bounded"),
    ("slack_from_the_last_best_entry", "float xi = c->tau * fminf(c->best[0].d, c->dnn);",
     "float xi = c->tau * fminf(dk, c->dnn);", "threshold_adds_slack_of_the_first"),
    ("user_query_takes_the_mean_dnn", "cache_init(&c, g, q, tau, g->stats[1], max_iter, -1);",
     "cache_init(&c, g, q, tau, g->stats[0], max_iter, -1);", "slack_uses_the_smaller or slack_is_bounded"),
    ("merge_takes_the_maximum_dnn", "cache_init(&c, g, q, p->tau_build, g->stats[0], p->max_iter, zb);",
     "cache_init(&c, g, q, p->tau_build, g->stats[1], p->max_iter, zb);", "merge_searches_from_the_top_segment"),
    ("visited_points_proposed_again", "  for (int i = 0; i < c->nv; i++) if (c->vis[i] == id) return 1;\n", "",
     "slack_uses_the_smaller"),
    # ---- capacities and limits (Alg. 2)
    ("iteration_limit_ignored", "  if (c->iter >= c->max_iter) return -1;\n", "", "iteration_limit_cuts"),
    ("iteration_limit_off_by_one", "if (c->iter >= c->max_iter) return -1;", "if (c->iter > c->max_iter) return -1;",
     "iteration_limit_cuts"),
    ("full_list_refuses_a_smaller_key", "if (*n == cap && !ent_less(e, a[cap - 1])) return;", "if (*n == cap) return;",
     "classical_best_first or full_prioq"),
    # ---- the layer change (Alg. 4)
    ("transform_drops_the_unpopped_prioq_entries",
     "  for (int i = 0; i < c->np; i++) if (!list_has(c->best, c->nb, c->pq[i].id)) all[na++] = c->pq[i];\n", "",
     "layer_change_keeps_unpopped"),
    ("transform_keeps_the_iteration_count", "  c->nv = c->vhead = 0;\n  c->iter = 0;\n", "  c->nv = c->vhead = 0;\n",
     "restarts_the_iteration_count"),
    ("transform_keeps_visited", "  c->nv = c->vhead = 0;\n  c->iter = 0;\n", "  c->iter = 0;\n", "layer_change_empties_visited"),
    # ---- hierarchical construction query (Alg. 3, Alg. 4, Alg. 6)
    ("segment_not_lifted_to_the_top_layer",
     "      for (int l = l_m; l < l_top; l++) seg /= g->g; /* top segment of z's sub-graph */\n", "",
     "merge_searches_from_the_top_segment"),
    ("descent_skips_the_middle_layers", "      for (int l = l_top - 1; l >= l_m; l--) {\n        cache_transform(&c, g->to_lower[l + 1]);",
     "      for (int l = l_m; l >= l_m; l--) {\n        cache_transform(&c, g->to_lower[l + 1]);", "descends_through_every_layer"),
    ("construction_query_admits_the_point_itself", "cache_init(&c, g, q, p->tau_build, g->stats[0], p->max_iter, zb);",
     "cache_init(&c, g, q, p->tau_build, g->stats[0], p->max_iter, -1);", "merge_searches_from_the_top_segment"),
    ("refinement_runs_bottom_up", "    for (int l_m = g->L - 2; l_m >= 0; l_m--) {\n      if ((rc = ggnn_ref_merge(g, g->L - 1, l_m, p)) != 0) return rc;",
     "    for (int l_m = 0; l_m <= g->L - 2; l_m++) {\n      if ((rc = ggnn_ref_merge(g, g->L - 1, l_m, p)) != 0) return rc;",
     "order_of_alg3_and_alg6"),
    # ---- symmetric linking (Alg. 5, Sec. 4.2.1)
    ("midpoint_weight_on_the_wrong_side", "float w = p->sym_constraint ? 0.4f : 0.0f;", "float w = p->sym_constraint ? 0.6f : 0.0f;",
     "shifted_midpoint"),
    ("radius_measured_from_z", "      c.radius = ggnn_ref_distance(q, row_ptr(g, xb), g->D, row_dtype(g), g->metric, g->lanes);",
     "      c.radius = ggnn_ref_distance(zv, row_ptr(g, xb), g->D, row_dtype(g), g->metric, g->lanes);", "shifted_midpoint"),
    ("slot_goes_to_the_farthest_request", "          if (ent_less(ew, ea)) wi = i;", "          if (ent_less(ea, ew)) wi = i;",
     "slots_go_to_the_closest"),
    ("losing_request_is_dropped", "        queue[qt] = loser; qt = (qt + 1) % qcap;\n", "", "slots_go_to_the_closest"),
    ("inverse_links_ignored_by_the_path_search", "        for (int i = 0; i < ninv[a]; i++) prop[np++] = inv[(int64_t)a * ksym + i];\n", "",
     "inverse_links_granted_in_earlier_rounds"),
    ("rows_offer_one_slot_less_than_k_sym", "        int cap = ksym - ninv[cand];", "        int cap = ksym - 1 - ninv[cand];",
     "path_inside_the_sphere"),
    ("granted_links_not_written_into_the_rows", "    for (int i = 0; i < nl; i++) row[o++] = links[i];\n", "",
     "path_inside_the_sphere or shifted_midpoint"),
    ("visited_list_stops_taking_entries_when_full",
     "    c->vis[c->vhead] = id;\n    c->vhead = (c->vhead + 1) % c->V;\n    if (c->nv < c->V) c->nv++;\n",
     "    if (c->nv < c->V) c->vis[c->nv++] = id;\n", "full_visited_list_forgets"),
    ("visited_list_overwrites_its_newest_entry", "    c->vhead = (c->vhead + 1) % c->V;\n",
     "    c->vhead = (c->vhead + 1 < c->V) ? c->vhead + 1 : c->V - 1;\n", "overwritten_in_order_of_arrival"),
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
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_oracle_handworked.py"), "-x", "-q",
                        "-k", pins, "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    # 1: a pin failed; a negative code: the mutant read outside its arrays and the run died, which no pin survives either
    assert r.returncode == 1 or r.returncode < 0, "the pins did not notice '%s':\n%s" % (name, r.stdout[-1500:])
    assert r.returncode < 0 or "failed" in r.stdout
