"""The pins must be able to fail: plant plausible mistakes in a copy of the oracle's C source (on the CPU), build
each, and check that the pin suites reject every one of them."""
import os
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
SRC = (ROOT / "oracle" / "la_oracle.c").read_text()

MUTANTS = {
    # attention
    "causal_off_by_one": ("const int64_t n = (int64_t)P + vis + i + 1;", "const int64_t n = (int64_t)P + vis + i;"),
    "sees_whole_branch": ("const int64_t n = (int64_t)P + vis + i + 1;", "const int64_t n = (int64_t)P + vis + L;"),
    "chain_not_counted": ("const int64_t n = (int64_t)P + vis + i + 1;", "const int64_t n = (int64_t)P + i + 1;"),
    "chain_of_wrong_request": ("int64_t base = (((int64_t)b * a->C + c) * a->Hkv + hk) * D;",
                               "int64_t base = (((int64_t)0 * a->C + c) * a->Hkv + hk) * D;"),
    "chain_vis_of_wrong_branch": ("  return c < a->chain_vis[(int64_t)b * a->gamma + g];",
                                  "  return c < a->chain_vis[(int64_t)b * a->gamma + 0];"),
    "tree_mask_of_wrong_branch": ("return (int)((a->seg_mask[(int64_t)b * a->gamma + g] >> seg) & 1u);",
                                  "return (int)((a->seg_mask[(int64_t)b * a->gamma + 0] >> seg) & 1u);"),
    "tree_segment_of_wrong_request": ("    const int seg = a->pool_seg[(int64_t)b * a->C + c];",
                                      "    const int seg = a->pool_seg[(int64_t)0 * a->C + c];"),
    "tree_mask_bit_off_by_one": ("return (int)((a->seg_mask[(int64_t)b * a->gamma + g] >> seg) & 1u);",
                                 "return (int)((a->seg_mask[(int64_t)b * a->gamma + g] >> (seg + 1)) & 1u);"),
    "tree_mask_truncated_to_32_bits": ("return (int)((a->seg_mask[(int64_t)b * a->gamma + g] >> seg) & 1u);",
                                       "return (int)(((uint32_t)a->seg_mask[(int64_t)b * a->gamma + g] >> (seg & 31)) & 1u);"),
    "visible_tokens_all_in_one_slot": ("    ++vis;\n", ""),
    "own_tokens_overwrite_chain": ("kcat[(int64_t)(P + vis + i) * D + d] = load_elem(a->k_branch",
                                   "kcat[(int64_t)(P + i) * D + d] = load_elem(a->k_branch"),
    "scale_dropped": ("    s *= a->scale;\n", ""),
    "gqa_head_map": ("h = hk * G + (int)(it % G);", "h = (int)(it % G) * Hkv + hk;"),
    "wrong_branch_kv": ("int64_t base = ((((int64_t)b * a->gamma + g) * a->L + i) * a->Hkv + hk) * D;",
                        "int64_t base = ((((int64_t)b * a->gamma + 0) * a->L + i) * a->Hkv + hk) * D;"),
    "block_table_ignored": ("int64_t phys = a->block_tables ?", "int64_t phys = 0 ?"),
    "block_offset": ("(j % a->block_size)) * D;", "((j + 1) % a->block_size)) * D;"),
    "k_scale_on_v": ("load_elem(a->v_cache, a->kv_dtype, base + d) * vs;", "load_elem(a->v_cache, a->kv_dtype, base + d) * ks;"),
    "no_max_subtraction_sign": ("w[j] = exp(w[j] - m);", "w[j] = exp(m - w[j]);"),
    "fp8_bias": ("ldexp(1.0 + (double)m / 8.0, e - 7)", "ldexp(1.0 + (double)m / 8.0, e - 8)"),
    "fp8_subnormal": ("ldexp((double)m / 8.0, -6)", "ldexp((double)m / 8.0, -7)"),
    # accept / resample
    "ratio_inverted": ("const int accept = (u * q[x] < p[x]);", "const int accept = (u * p[x] < q[x]);"),
    "no_stop_at_rejection": ("        n = i;\n        break;", "        n = i;"),
    "residual_sign": ("r[v] = p[v] - q[v];", "r[v] = q[v] - p[v];"),
    "resample_from_p": ("        if (r[v] < 0.0) r[v] = 0.0;\n", "        r[v] = p[v];\n"),
    "bonus_from_wrong_row": ("((int64_t)nb * (K + 1) + K) * V, V, temperature, r);",
                             "((int64_t)nb * (K + 1) + K - 1) * V, V, temperature, r);"),
    "cdf_not_strict_start": ("      if (c > thr) {", "      if (c >= thr) {"),
    "temperature_ignored": ("p[v] = load_elem(logits, dtype, base + v) / temperature;",
                            "p[v] = load_elem(logits, dtype, base + v);"),
    "topk_one_too_many": ("    kept = top_k;\n", "    kept = top_k + 1;\n"),
    "topk_splits_ties": ("    while (kept < V && r[kept].v == r[top_k - 1].v) ++kept; /* ties with the k-th largest stay */\n", ""),
    "topp_ignores_topk_mass": ("    const double T = top_p * zk;\n", "    const double T = top_p;\n"),
    "topp_splits_ties": ("      while (e < kept && r[e].v == r[j].v) gm += r[e++].v;\n", "      gm += r[e++].v;\n"),
    "topp_keeps_one_group_less": ("      if (!(M < T)) break; /* the tokens of this value have mass >= T above them */\n",
                                  "      if (!(M + r[j].v < T)) break;\n"),
    "warp_not_renormalised": ("  for (int j = 0; j < kept; ++j) p[r[j].id] = r[j].v / z;\n",
                              "  for (int j = 0; j < kept; ++j) p[r[j].id] = r[j].v;\n"),
    "warp_skipped_for_bonus_row": ("      if (warp_row(r, V, top_k, top_p, &wm_row)) failed = 1;\n", "      wm_row = INFINITY;\n"),
    "point_mass_keeps_x": ("        q[x] = 1.0;\n", "        q[x] = 0.0;\n"),
    "point_mass_on_wrong_token": ("        q[x] = 1.0;\n", "        q[(x + 1) % V] = 1.0;\n"),
    "draft_row_index": ("softmax_row(draft_logits, logits_dtype, ((int64_t)nb * K + i) * V",
                        "softmax_row(draft_logits, logits_dtype, ((int64_t)nb * K + 0) * V"),
}

# KV commit: checked by its own pin file only
COMMIT_MUTANTS = {
    "commit_position_off_by_one": ("block_tables, prefix_lens[b], k_branch, v_branch, C, k_chain, v_chain, rows, n_chain[b],",
                                   "block_tables, prefix_lens[b] + 1, k_branch, v_branch, C, k_chain, v_chain, rows, n_chain[b],"),
    "commit_own_before_chain": ("    const int from_drafted = t < n_drafted;",
                                "    const int from_drafted = t >= n_own;"),
    "commit_own_index_not_rebased": ("        const int i = t - n_drafted;", "        const int i = t;"),
    "commit_wrong_branch": ("src = ((((int64_t)b * gamma + src_branch) * L + i) * Hkv + hk) * D;",
                            "src = ((((int64_t)b * gamma + 0) * L + i) * Hkv + hk) * D;"),
    "commit_chain_of_wrong_request": ("        src = (((int64_t)b * C + drafted[t]) * Hkv + hk) * D;",
                                      "        src = (((int64_t)0 * C + drafted[t]) * Hkv + hk) * D;"),
    "commit_chain_reversed": ("  for (int c = 0; c < C; ++c) rows[c] = c;", "  for (int c = 0; c < C; ++c) rows[c] = C - 1 - c;"),
    "commit_block_table_ignored": ("    const int64_t phys = block_tables ? (int64_t)block_tables[(int64_t)b * max_blocks + logical_block]",
                                   "    const int64_t phys = 0 ? (int64_t)block_tables[(int64_t)b * max_blocks + logical_block]"),
    "commit_slot_in_block": ("const int64_t dst = ((phys * Hkv + hk) * block_size + (pos % block_size)) * D;",
                             "const int64_t dst = ((phys * Hkv + hk) * block_size + (t % block_size)) * D;"),
    "commit_v_from_k": ("if (commit_row(vs, br_dtype, src, v_cache, kv_dtype, dst, D, v_scale, hk)) return 2;",
                        "if (commit_row(ks, br_dtype, src, v_cache, kv_dtype, dst, D, v_scale, hk)) return 2;"),
    "commit_k_scale_on_v": ("if (commit_row(vs, br_dtype, src, v_cache, kv_dtype, dst, D, v_scale, hk)) return 2;",
                            "if (commit_row(vs, br_dtype, src, v_cache, kv_dtype, dst, D, k_scale, hk)) return 2;"),
    "commit_new_len_without_chain": ("    new_prefix_lens[b] = prefix_lens[b] + n_chain[b] + n_own[b];",
                                     "    new_prefix_lens[b] = prefix_lens[b] + n_own[b];"),
    "tree_commit_keeps_the_discarded": ("      if ((commit_mask[b] >> pool_seg[(int64_t)b * C + c]) & 1u) rows[kept++] = c;",
                                        "      if (1) rows[kept++] = c;"),
    "tree_commit_keeps_the_complement": ("      if ((commit_mask[b] >> pool_seg[(int64_t)b * C + c]) & 1u) rows[kept++] = c;",
                                         "      if (!((commit_mask[b] >> pool_seg[(int64_t)b * C + c]) & 1u)) rows[kept++] = c;"),
    "tree_commit_mask_of_request_0": ("      if ((commit_mask[b] >> pool_seg[(int64_t)b * C + c]) & 1u) rows[kept++] = c;",
                                      "      if ((commit_mask[0] >> pool_seg[(int64_t)b * C + c]) & 1u) rows[kept++] = c;"),
    "tree_commit_nodes_of_request_0": ("      if ((commit_mask[b] >> pool_seg[(int64_t)b * C + c]) & 1u) rows[kept++] = c;",
                                       "      if ((commit_mask[b] >> pool_seg[(int64_t)0 * C + c]) & 1u) rows[kept++] = c;"),
    "tree_commit_mask_truncated_to_32_bits": ("      if ((commit_mask[b] >> pool_seg[(int64_t)b * C + c]) & 1u) rows[kept++] = c;",
                                              "      if (((uint32_t)commit_mask[b] >> (pool_seg[(int64_t)b * C + c] & 31)) & 1u) rows[kept++] = c;"),
    "tree_commit_rows_not_the_kept_ones": ("      if ((commit_mask[b] >> pool_seg[(int64_t)b * C + c]) & 1u) rows[kept++] = c;",
                                           "      if ((commit_mask[b] >> pool_seg[(int64_t)b * C + c]) & 1u) rows[kept] = kept, ++kept;"),
    "tree_commit_new_len_without_pool": ("    new_prefix_lens[b] = prefix_lens[b] + kept + n_own[b];",
                                         "    new_prefix_lens[b] = prefix_lens[b] + n_own[b];"),
    "quantiser_multiplies": ("      const float y = x / s; /* fp32 quotient, correctly rounded */",
                             "      const float y = x * s;"),
    "quantiser_scale_of_head_0": ("    const float s = scale ? scale[hk] : 1.0f;", "    const float s = scale ? scale[0] : 1.0f;"),
    "quantiser_ties_up": ("    if (d < best_d || (d == best_d && (code & 1) == 0)) {", "    if (d <= best_d) {"),
    "quantiser_ties_down": ("    if (d < best_d || (d == best_d && (code & 1) == 0)) {", "    if (d < best_d) {"),
    "quantiser_no_saturation": ("  if (a > 448.0) best = 126;\n", "  if (a > 448.0) best = 127;\n"),
    "quantiser_drops_sign": ("  return (uint8_t)(best | (signbit(y) ? 0x80 : 0));", "  return (uint8_t)best;"),
}
# each mutant is run against the pin file of the function it sits in (the storage widening is used by both)
_names = list(MUTANTS)
_first_accept = _names.index("ratio_inverted")
SUITES = {name: ["tests/test_oracle_attention.py"] for name in _names[:_first_accept]}
SUITES.update({name: ["tests/test_oracle_accept.py"] for name in _names[_first_accept:]})
SUITES.update({name: ["tests/test_oracle_commit.py"] for name in COMMIT_MUTANTS})
MUTANTS.update(COMMIT_MUTANTS)


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_reject_mutant(name, tmp_path):
    old, new = MUTANTS[name]
    assert SRC.count(old) == 1, f"mutation site for {name} not found exactly once"
    src = tmp_path / "mutant.c"
    lib = tmp_path / "libmutant.so"
    src.write_text(SRC.replace(old, new))
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-w", "-o", str(lib), str(src), "-lm"], check=True)
    env = dict(os.environ, LA_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        *SUITES[name]],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 1, f"mutant {name} was not caught:\n{r.stdout[-2000:]}"


# ---- the planner oracle is Python: same idea, on its source text ------------------------------------------------
PLANNER_SRC = (ROOT / "oracle" / "planner.py").read_text()
PLANNER_MUTANTS = {
    "first_rejection_returns_last": ("        if not ok:\n            return j\n", "        if not ok:\n            last = j\n"),
    "all_accepted_off_by_one": ("    return len(verdicts)\n", "    return len(verdicts) - 1\n"),
    "tree_walk_takes_last_matching": ("            here = min(matching)\n", "            here = max(matching)\n"),
    "tree_walk_stops_after_one_step": ("            here = min(matching)\n            accepted.append(here)\n",
                                       "            here = min(matching)\n            accepted.append(here)\n            break\n"),
    "tree_walk_looks_at_all_nodes": ("alternatives = [n for n in range(len(parent)) if parent[n] == here]",
                                     "alternatives = [n for n in range(len(parent)) if parent[n] >= here]"),
    "tree_walk_branch_of_parent": ("out.append((len(accepted), here + 1, sum(1 << n for n in accepted), int(own[here + 1])))",
                                   "out.append((len(accepted), here, sum(1 << n for n in accepted), int(own[here + 1])))"),
    "tree_walk_own_of_root": ("out.append((len(accepted), here + 1, sum(1 << n for n in accepted), int(own[here + 1])))",
                              "out.append((len(accepted), here + 1, sum(1 << n for n in accepted), int(own[0])))"),
    "tree_walk_mask_is_depth_bits": ("out.append((len(accepted), here + 1, sum(1 << n for n in accepted), int(own[here + 1])))",
                                     "out.append((len(accepted), here + 1, (1 << len(accepted)) - 1, int(own[here + 1])))"),
    "output_keeps_own_of_next_branch": ("out.append((j, j, int(vis[j]), int(own[j])))",
                                        "out.append((j, j, int(vis[j]), int(own[min(j + 1, len(own) - 1)])))"),
    "output_chain_of_previous_branch": ("out.append((j, j, int(vis[j]), int(own[j])))",
                                        "out.append((j, j, int(vis[max(j - 1, 0)]), int(own[j])))"),
    "sync_counts_k_drafts": ("    emitted = _expect(alpha, lambda x: min(x, k - 1) + 1)\n    return emitted / ((k - 1) * c + 1.0)",
                             "    emitted = _expect(alpha, lambda x: min(x, k - 1) + 1)\n    return emitted / (k * c + 1.0)"),
    "sync_emits_up_to_k_drafts": ("lambda x: min(x, k - 1) + 1)", "lambda x: min(x, k) + 1)"),
    "async_floor_instead_of_ceil": ("lambda x: -(-(x + 1) // k) + c * (x % k))", "lambda x: (x + 1) // k + c * (x % k))"),
    "async_mod_of_x_plus_1": ("lambda x: -(-(x + 1) // k) + c * (x % k))", "lambda x: -(-(x + 1) // k) + c * ((x + 1) % k))"),
    "async_case_switch_strict": ("    if k >= depth_limit(c):", "    if k > depth_limit(c):"),
    "depth_limit_floor": ("    return int(math.ceil(1.0 / c))", "    return int(math.floor(1.0 / c))"),
    "geometric_law_shifted": ("    total, n, w = 0.0, 0, 1.0 - alpha", "    total, n, w = 0.0, 1, 1.0 - alpha"),
    "async_budget_uses_k1": ("    return min(depth_limit(c1), k1) if asynchronous else k1", "    return k1"),
    "budget_is_a_sum": ("            if parallel_dim_f(c1, k1, asynchronous) * k2 > budget:",
                        "            if parallel_dim_f(c1, k1, asynchronous) + k2 > budget:"),
    "plan_minimises": ("            if best is None or h > best[2]:", "            if best is None or h < best[2]:"),
    "token_level_uses_step_parameters": ("    g = {k2: speedup_sync(alpha2, c2, k2)", "    g = {k2: speedup_sync(alpha1, c1, k2)"),
}


@pytest.mark.parametrize("name", sorted(PLANNER_MUTANTS))
def test_planner_pins_reject_mutant(name, tmp_path):
    old, new = PLANNER_MUTANTS[name]
    assert PLANNER_SRC.count(old) == 1, f"mutation site for {name} not found exactly once"
    src = tmp_path / "planner_mutant.py"
    src.write_text(PLANNER_SRC.replace(old, new))
    env = dict(os.environ, LA_ORACLE_PLANNER_SRC=str(src))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        "tests/test_oracle_planner.py"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 1, f"mutant {name} was not caught:\n{r.stdout[-2000:]}"
