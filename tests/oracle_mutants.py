"""Planted mistakes for the oracle's own pins.

Each entry rewrites one spot of `oracle/baklava_oracle.py` the way a plausible slip would (a wrong
scale, swapped operands, an off-by-one window, a tie broken the other way ...) and names the pin
files that must notice.  `install(name)` builds the altered module in memory and registers it under
the oracle's module name, so that the unchanged pin tests run against it; nothing on disk changes
and nothing outside the CPU test-suite uses this."""
import os
import sys
import types

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_PATH = os.path.join(ROOT, "oracle", "baklava_oracle.py")

ALLOC, ATTN, COMPACT = "tests/test_oracle_alloc.py", "tests/test_oracle_attention.py", "tests/test_oracle_compact.py"
PROFILE, PREFILL, LAYER = "tests/test_oracle_profile.py", "tests/test_oracle_prefill.py", "tests/test_oracle_layer.py"

# name -> ([(old text, new text), ...], [pin files])
MUTANTS = {
    # ---- proportional allocation
    "prop_leftover_to_smallest_remainders": (
        [("elig.sort(key=lambda i: ((lam * w[i]) & (one - 1), w[i], -i), reverse=True)",
          "elig.sort(key=lambda i: ((lam * w[i]) & (one - 1), w[i], -i))")], [ALLOC]),
    "prop_no_upper_clip": ([("return lo if x < lo else (hi if x > hi else x)", "return lo if x < lo else x")], [ALLOC]),
    "prop_leftover_may_exceed_hi": ([("elig = [i for i in range(m) if lo <= x[i] < hi]",
                                      "elig = [i for i in range(m) if lo <= x[i] <= hi]")], [ALLOC]),
    "prop_weights_not_monotone": ([("w = [max(1, int(math.floor((v / top) * float(one)))) for v in imp]",
                                    "w = [max(1, int(math.floor((top / v) * 1024.0))) for v in imp]")], [ALLOC]),
    # ---- Algorithm 2
    "thr_low_set_includes_threshold": ([("low = [i for i in range(m) if imp[i] < t]",
                                         "low = [i for i in range(m) if imp[i] <= t]")], [ALLOC]),
    "thr_all_high_caches_receive": ([("    k = min(n, m - n)\n", "    k = m - n\n")], [ALLOC]),
    "thr_least_important_receive": ([("high.sort(key=lambda i: (-imp[i], i))", "high.sort(key=lambda i: (imp[i], i))")], [ALLOC]),
    "thr_remainder_to_last": ([("base + (1 if rank < rem else 0)", "base + (1 if rank >= k - rem else 0)")], [ALLOC]),
    "thr_reduction_rounds_up": ([("d = int(math.floor(r * size[i]))", "d = int(math.ceil(r * size[i]))")], [ALLOC]),
    "thr_reduction_is_amount": ([("d = int(math.floor(r * size[i]))", "d = min(size[i], int(math.floor(r * 100)))")], [ALLOC]),
    # ---- layout
    "layout_inclusive_prefix": ([("                off.append(total)\n                cap.append(c)\n                total += c",
                                  "                cap.append(c)\n                total += c\n                off.append(total)")], [ALLOC]),
    "layout_no_slack": ([("c = int(budget[l * Hkv + h]) + slack", "c = int(budget[l * Hkv + h])")], [ALLOC]),
    "layout_budget_per_sequence": ([("c = int(budget[l * Hkv + h]) + slack", "c = int(budget[(l * Hkv + h + b) % len(budget)]) + slack")], [ALLOC]),
    # ---- decode attention
    "attn_scale_by_D": ([("s = (K @ q[g]) / math.sqrt(D)       # s_j", "s = (K @ q[g]) / D       # s_j")], [ATTN]),
    "attn_no_scale": ([("s = (K @ q[g]) / math.sqrt(D)       # s_j", "s = (K @ q[g])       # s_j")], [ATTN]),
    "attn_values_are_keys": ([("out[g] = p[g] @ V", "out[g] = p[g] @ K")], [ATTN]),
    "attn_logits_from_values": ([("s = (K @ q[g]) / math.sqrt(D)       # s_j", "s = (V @ q[g]) / math.sqrt(D)       # s_j")], [ATTN]),
    "attn_weights_not_normalised": ([("p[g] = e / np.sum(e)", "p[g] = e / np.max(e)")], [ATTN]),
    "attn_one_query_head_for_all": ([("s = (K @ q[g]) / math.sqrt(D)       # s_j", "s = (K @ q[0]) / math.sqrt(D)       # s_j")], [ATTN]),
    # ---- score accumulation, append, step order
    "score_mean_over_heads": ([("+ np.sum(p, axis=0)", "+ np.mean(p, axis=0)")], [ATTN, PREFILL]),
    "score_max_over_heads": ([("+ np.sum(p, axis=0)", "+ np.max(p, axis=0)")], [ATTN, PREFILL]),
    "append_score_starts_at_one": ([("self.score = np.append(self.score, 0.0)", "self.score = np.append(self.score, 1.0)")], [ATTN, COMPACT]),
    "append_row_goes_first": ([("self.K = np.vstack([self.K, np.asarray(k_row, dtype=np.float64)[None, :]])",
                                "self.K = np.vstack([np.asarray(k_row, dtype=np.float64)[None, :], self.K])")], [ATTN, COMPACT]),
    "step_evicts_one_step_early": ([("if interval > 0 and step_index % interval == 0:",
                                     "if interval > 0 and (step_index + 1) % interval == 0:")], [ATTN, COMPACT]),
    "step_attends_before_append": ([("    if k_new is not None:\n        cache.append(k_new, v_new, token_pos)\n    out, p = decode_attn(q, cache.K, cache.V)",
                                     "    out, p = decode_attn(q, cache.K, cache.V)\n    if k_new is not None:\n        cache.append(k_new, v_new, token_pos)\n        p = np.concatenate([p, np.zeros((p.shape[0], 1))], axis=1)")], [ATTN]),
    # ---- eviction
    "evict_ties_to_newer_row": ([("mid.sort(key=lambda j: (-float(s32[j]), j))", "mid.sort(key=lambda j: (-float(s32[j]), -j))")], [COMPACT]),
    "evict_keeps_lowest_scores": ([("mid.sort(key=lambda j: (-float(s32[j]), j))", "mid.sort(key=lambda j: (float(s32[j]), j))")], [COMPACT]),
    "evict_recent_window_shifted": ([("kept = list(range(sink)) + mid[:k] + list(range(n - recent, n))",
                                      "kept = list(range(sink)) + mid[:k] + list(range(n - recent - 1, n - 1))")], [COMPACT]),
    "evict_sink_rows_compete": ([("mid = list(range(sink, n - recent))\n", "mid = list(range(0, n - recent))\n"),
                                 ("kept = list(range(sink)) + mid[:k] +", "kept = mid[:k + sink] +")], [COMPACT]),
    "evict_scores_compared_in_fp64": ([("s32 = np.asarray(score[:n], dtype=np.float32)", "s32 = np.asarray(score[:n], dtype=np.float64)")], [COMPACT]),
    "evict_streaming_keeps_a_scored_row": ([("        recent = budget - sink\n", "        recent = budget - sink - 1\n")], [COMPACT]),
    "evict_survivors_reordered": ([("    kept.sort()\n    return kept", "    return kept")], [COMPACT]),
    "evict_scores_not_moved": ([("        self.score = self.score[kept]\n", "        self.score = self.score[: len(kept)]\n")], [COMPACT, ATTN]),
    # ---- Algorithm 1
    "sim_not_causal": ([("s = (K[: t + 1] @ Q[t]) * scale\n        w = np.exp(s - s.max())\n        out = (w / w.sum()) @ V[: t + 1]",
                         "s = (K @ Q[t]) * scale\n        w = np.exp(s - s.max())\n        out = (w / w.sum()) @ V")], [PROFILE]),
    "sim_mask_excludes_own_token": ([("s = (K[: t + 1] @ Q[t]) * scale\n        w = np.exp(s - s.max())\n        out = (w / w.sum()) @ V[: t + 1]",
                                      "s = (K[: max(t, 1)] @ Q[t]) * scale\n        w = np.exp(s - s.max())\n        out = (w / w.sum()) @ V[: max(t, 1)]")], [PROFILE]),
    "sim_no_scale": ([("    cos = np.empty(T, dtype=np.float64)\n    scale = 1.0 / math.sqrt(D)", "    cos = np.empty(T, dtype=np.float64)\n    scale = 1.0")], [PROFILE]),
    "sim_cosine_with_key_row": ([("cos[t] = float(V[t] @ out) / denom", "cos[t] = float(K[t] @ out) / denom")], [PROFILE]),
    "sim_not_normalised_by_value_norm": ([("denom = max(float(np.linalg.norm(V[t]) * np.linalg.norm(out)), COS_EPS)",
                                           "denom = max(float(np.linalg.norm(out) * np.linalg.norm(out)), COS_EPS)")], [PROFILE]),
    "sim_sum_instead_of_mean": ([("    return float(cos.mean()), cos\n\n\ndef kv_importance", "    return float(cos.sum()), cos\n\n\ndef kv_importance")], [PROFILE]),
    "imp_no_complement": ([("return 1.0 - (grouped + 1.0) / 2.0", "return (grouped + 1.0) / 2.0")], [PROFILE]),
    "imp_no_map_to_unit_interval": ([("return 1.0 - (grouped + 1.0) / 2.0", "return 1.0 - grouped")], [PROFILE]),
    "imp_groups_strided": ([("grouped = s.reshape(L, Hq // G, G).mean(axis=2)", "grouped = s.reshape(L, G, Hq // G).mean(axis=1)")], [PROFILE]),
    # ---- scores of a whole prompt
    "prefill_not_causal": ([("            s = (K[: t + 1] @ Q[g, t]) * scale\n            w = np.exp(s - s.max())\n            score[: t + 1] += w / w.sum()",
                             "            s = (K @ Q[g, t]) * scale\n            w = np.exp(s - s.max())\n            score += w / w.sum()")], [PREFILL]),
    "prefill_no_scale": ([("    score = np.zeros(T, dtype=np.float64)\n    scale = 1.0 / math.sqrt(D)", "    score = np.zeros(T, dtype=np.float64)\n    scale = 1.0")], [PREFILL]),
    "prefill_heads_averaged": ([("            score[: t + 1] += w / w.sum()\n    return score", "            score[: t + 1] += w / w.sum()\n    return score / G")], [PREFILL]),
    "prefill_rows_not_normalised": ([("            score[: t + 1] += w / w.sum()", "            score[: t + 1] += w")], [PREFILL]),
    # ---- layer heuristic and the two-level allocation
    "layer_cosine_norm_of_input_only": ([("denom = max(float(np.linalg.norm(A[t]) * np.linalg.norm(Bm[t])), COS_EPS)",
                                          "denom = max(float(np.linalg.norm(A[t]) * np.linalg.norm(A[t])), COS_EPS)")], [LAYER]),
    "layer_dot_with_itself": ([("cos[t] = float(A[t] @ Bm[t]) / denom", "cos[t] = float(Bm[t] @ Bm[t]) / denom")], [LAYER]),
    "two_level_pool_bounds_per_cache": ([("pools = alloc_proportional(layer_importance, global_budget, Hkv * lo, Hkv * hi)",
                                          "pools = alloc_proportional(layer_importance, global_budget, lo, Hkv * hi)")], [LAYER]),
    "two_level_remainder_to_least_important": ([("order = sorted(range(Hkv), key=lambda i: (-himp[l, i], i))",
                                                 "order = sorted(range(Hkv), key=lambda i: (himp[l, i], i))")], [LAYER]),
    "two_level_skips_algorithm_2": ([("out.extend(alloc_threshold(himp[l].tolist(), size, t, r))", "out.extend(size)")], [LAYER]),
    "two_level_equal_pools": ([("pools = alloc_proportional(layer_importance, global_budget, Hkv * lo, Hkv * hi)",
                                "pools = alloc_proportional([1.0] * L, global_budget, Hkv * lo, Hkv * hi)")], [LAYER]),
    # ---- further spots
    "evict_pos_not_moved": ([("        self.pos = self.pos[kept]\n", "        self.pos = self.pos[: len(kept)]\n")], [COMPACT, ATTN]),
    "evict_values_not_moved": ([("        self.V = self.V[kept]\n", "        self.V = self.V[: len(kept)]\n")], [COMPACT, ATTN]),
    "thr_topk_ties_to_higher_index": ([("high.sort(key=lambda i: (-imp[i], i))", "high.sort(key=lambda i: (-imp[i], -i))")], [ALLOC]),
    "layout_heads_outer_loop": ([("        for b in range(batch):\n            for h in range(Hkv):\n",
                                  "        for h in range(Hkv):\n            for b in range(batch):\n")], [ALLOC]),
    "imp_group_max": ([("grouped = s.reshape(L, Hq // G, G).mean(axis=2)", "grouped = s.reshape(L, Hq // G, G).max(axis=2)")], [PROFILE]),
    "prefill_first_head_only": ([("            s = (K[: t + 1] @ Q[g, t]) * scale\n", "            s = (K[: t + 1] @ Q[0, t]) * scale\n")], [PREFILL]),
    "layer_mean_is_last_token": ([("    return float(cos.mean()), cos\n\n\ndef alloc_two_level", "    return float(cos[-1]), cos\n\n\ndef alloc_two_level")], [LAYER]),
    "score_not_cumulative": ([("return np.asarray(score, dtype=np.float64) + np.sum(p, axis=0)", "return np.sum(p, axis=0)")], [ATTN, PREFILL]),
    "sim_keys_and_values_swapped": ([("s = (K[: t + 1] @ Q[t]) * scale\n        w = np.exp(s - s.max())\n        out = (w / w.sum()) @ V[: t + 1]",
                                      "s = (V[: t + 1] @ Q[t]) * scale\n        w = np.exp(s - s.max())\n        out = (w / w.sum()) @ K[: t + 1]")], [PROFILE]),
    "prop_budget_from_unclipped_share": ([("    b = [clip(xi) for xi in x]\n", "    b = [max(lo, xi) for xi in x]\n")], [ALLOC]),
    "evict_nothing_when_over_budget_by_one": ([("    if n <= budget:\n        return list(range(n))", "    if n <= budget + 1:\n        return list(range(n))")], [COMPACT]),
    "two_level_threshold_ignores_layer": ([("out.extend(alloc_threshold(himp[l].tolist(), size, t, r))", "out.extend(alloc_threshold(himp[0].tolist(), size, t, r))")], [LAYER]),
}


def mutated_source(name: str) -> str:
    src = open(ORACLE_PATH).read()
    for old, new in MUTANTS[name][0]:
        if src.count(old) != 1:
            raise ValueError(f"mutant {name}: the text to replace occurs {src.count(old)} times in the oracle")
        src = src.replace(old, new)
    return src


def install(name: str) -> None:
    """Register the altered oracle as `oracle.baklava_oracle` for this process."""
    import oracle  # the package itself stays as it is
    mod = types.ModuleType("oracle.baklava_oracle")
    mod.__file__ = ORACLE_PATH
    exec(compile(mutated_source(name), ORACLE_PATH + f" [mutant {name}]", "exec"), mod.__dict__)
    sys.modules["oracle.baklava_oracle"] = mod
    oracle.baklava_oracle = mod
