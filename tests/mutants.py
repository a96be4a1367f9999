"""Copies of the oracle's C source with one planted mistake each (helper of the mutation tests).

A mutant is a single textual change of the kind a slip would make: a dropped term, a wrong sign,
index, constant or inequality, swapped operands.  The mistakes live in the oracle only; they are
compiled on the CPU into temporary libraries that ``oracle.rc_oracle`` loads when the environment
variable RC_ORACLE_LIB names one.
"""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "rc_oracle.c")

# (name, text to find, replacement, which occurrence (0-based) or None for all)
MUTANTS = [
    ("f16_exponent_bias", "ldexp((double)(1024 + m), e - 25)", "ldexp((double)(1024 + m), e - 24)", 0),
    ("f16_subnormal_scale", "ldexp((double)m, -24)", "ldexp((double)m, -25)", 0),
    ("f16_sign_dropped", "return sign ? -v : v;", "return v;", 0),
    ("bf16_shift", "(uint32_t)b << 16", "(uint32_t)b << 15", 0),
    ("layout_head_innermost", "((int64_t)t * H + h) * Dh + d", "((int64_t)t * Dh + d) * H + h", 0),
    ("norms_k_and_v_swapped", "const uint16_t* src = (which ? v : k) +", "const uint16_t* src = (which ? k : v) +", 0),
    ("norms_layer_stride_ignored", "(which ? v : k) + (int64_t)l * layer_stride + b * D;", "(which ? v : k) + b * D;", 0),
    ("score_pairs_query_index", "decode_block(dtype, kq + (int64_t)li[i] * q_layer_stride + (int64_t)qi[i] * D, D, buf);",
     "decode_block(dtype, kq + (int64_t)li[i] * q_layer_stride + (int64_t)pi[i] * D, D, buf);", 0),
    ("score_pairs_layer_ignored", "decode_block(dtype, vp + (int64_t)li[i] * p_layer_stride + (int64_t)pi[i] * D, D, buf + 3 * D);",
     "decode_block(dtype, vp + (int64_t)pi[i] * D, D, buf + 3 * D);", 0),
    ("match_head_v_uses_k_norm", "qvn[q * NH + h], pvn[h]);", "qkn[q * NH + h], pvn[h]);", 0),
    ("match_query_layer_stride_ignored", "decode_block(dtype, vq + (int64_t)l * q_layer_stride + q * D, D, qv + q * D);\n      for (int h = 0; h < NH; ++h)",
     "decode_block(dtype, vq + q * D, D, qv + q * D);\n      for (int h = 0; h < NH; ++h)", 0),
    ("layer_mean_pool_layer_stride_ignored", "decode_block(dtype, vp + (int64_t)l * p_layer_stride + p * D, D, pv);\n      for (int64_t q = 0; q < Q; ++q) {\n        double sk",
     "decode_block(dtype, vp + p * D, D, pv);\n      for (int64_t q = 0; q < Q; ++q) {\n        double sk", 0),
    ("layer_mean_runner_up_not_raised", "else if (d < sd) sd = d;", "", 0),
    ("cand_dist_query_layer_ignored", "decode_block(dtype, kq + (int64_t)l * q_layer_stride + q * D, D, buf);\n          decode_block(dtype, vq + (int64_t)l * q_layer_stride + q * D, D, buf + D);\n          decode_block(dtype, kp",
     "decode_block(dtype, kq + q * D, D, buf);\n          decode_block(dtype, vq + (int64_t)l * q_layer_stride + q * D, D, buf + D);\n          decode_block(dtype, kp", 0),
    ("admit_layers_after_first_not_copied", "    for (int l = 0; l < L; ++l) {\n      memcpy(kp", "    for (int l = 0; l < 1; ++l) {\n      memcpy(kp", 0),
    ("admit_count_includes_rejected", "    if (next >= P) continue; /* pool full */", "    if (next >= P) { ++count; continue; }", 0),
    ("remap_refcounts_not_carried_over", "refcount_out[(int64_t)l * NB + b] = refcount_in[(int64_t)l * NB + b];", "refcount_out[(int64_t)l * NB + b] = 0;", 0),
    ("remap_out_of_range_entry_clamped", "      } else {\n        tout[e] = b;\n      }", "      } else {\n        tout[e] = -1;\n      }", 0),
    ("norm_head_filter_inverted", "if (head >= 0 && h != head) continue;", "if (head >= 0 && h == head) continue;", 0),
    ("dot_head_filter_dropped", "if (head >= 0 && h != head) continue;", "", 1),
    ("touch_out_of_range_clamped", "if (slots[i] >= 0 && slots[i] < P) array[slots[i]] = value;",
     "array[slots[i] < 0 ? 0 : slots[i] >= P ? P - 1 : slots[i]] = value;", 0),
    ("release_without_multiplicity", "if (ids[i] >= 0 && ids[i] < NB) refcount[ids[i]] -= 1;",
     "if (ids[i] >= 0 && ids[i] < NB && (i == 0 || ids[i] != ids[i - 1])) refcount[ids[i]] -= 1;", 0),
    ("evict_referenced_slots_too", "if (!live[p] || (refcount && refcount[p] != 0)) continue;", "if (!live[p]) continue;", 0),
    ("evict_most_recently_used", "last_used[p] < last_used[victim]", "last_used[p] > last_used[victim]", 0),
    ("evict_tie_to_highest_slot", "last_used[p] < last_used[victim]", "last_used[p] <= last_used[victim]", 0),
    ("evict_ignores_free_slots", "for (int64_t p = 0; p < P; ++p) free_slots += !live[p];", "", 0),
    ("evict_counts_matched_queries", "wanted += match_idx[q] < 0;", "wanted += 1;", 0),
    ("evict_extra_wanted_dropped", "int64_t wanted = extra_wanted, free_slots = 0, evicted = 0;",
     "int64_t wanted = 0, free_slots = 0, evicted = 0;", 0),
    ("norm_not_squared", "acc += a * a;", "acc += fabs(a);", 0),
    ("cosine_without_sqrt", "return xy / sqrt(xx * yy);", "return xy / (xx * yy);", 0),
    ("cosine_zero_norm_and", "if (xx == 0.0 || yy == 0.0) return 0.0;", "if (xx == 0.0 && yy == 0.0) return 0.0;", 0),
    ("pair_score_v_dropped", "return 0.5 * (ck + cv);", "return 0.5 * (ck + ck);", 0),
    ("pair_score_not_halved", "return 0.5 * (ck + cv);", "return (ck + cv);", 0),
    ("pair_score_head_max", "if (sh < s) s = sh;\n  }\n  return s;", "if (sh > s || h == 0) s = sh;\n  }\n  return s;", 0),
    ("match_k_uses_v_norm", "cosine(dot(qk + q * D, pk, T, H, Dh, -1), qkn[q], pkn[0])",
     "cosine(dot(qk + q * D, pk, T, H, Dh, -1), qvn[q], pkn[0])", 0),
    ("match_v_uses_k_tensor", "cosine(dot(qv + q * D, pv, T, H, Dh, -1), qvn[q], pvn[0])",
     "cosine(dot(qv + q * D, pk, T, H, Dh, -1), qvn[q], pvn[0])", 0),
    ("match_head_norm_index", "qkn[q * NH + h], pkn[h])", "qkn[q * NH], pkn[h])", 0),
    ("match_head_mean_not_min", "            if (sh < s) s = sh;", "            s = (h == 0) ? sh / H : s + sh / H;", 0),
    ("match_dead_blocks_not_skipped", "if (live && !live[(int64_t)l * P + p]) continue;", "", 0),
    ("match_tie_highest_index", "if (s > bs) { ss = bs; bs = s; bi = (int32_t)p; }", "if (s >= bs) { ss = bs; bs = s; bi = (int32_t)p; }", 0),
    ("match_runner_up_not_demoted", "if (s > bs) { ss = bs; bs = s; bi = (int32_t)p; }", "if (s > bs) { bs = s; bi = (int32_t)p; }", 0),
    ("match_runner_up_not_raised", "else if (s > ss) ss = s;", "", 0),
    ("match_threshold_strict", "(bi >= 0 && bs >= tau) ? bi : -1;\n    }\n    if (scores_out)", "(bi >= 0 && bs > tau) ? bi : -1;\n    }\n    if (scores_out)", 0),
    ("match_layer_stride_ignored", "decode_block(dtype, kp + (int64_t)l * p_layer_stride + p * D, D, pk);\n      decode_block(dtype, vp + (int64_t)l * p_layer_stride + p * D, D, pv);\n      for (int h = 0; h < NH; ++h)",
     "decode_block(dtype, kp + p * D, D, pk);\n      decode_block(dtype, vp + p * D, D, pv);\n      for (int h = 0; h < NH; ++h)", 0),
    ("candidates_tie_highest_index", "if (s > bs || (s == bs && pidx < bi)) { bs = s; bi = pidx; }", "if (s >= bs) { bs = s; bi = pidx; }", 0),
    ("candidates_dead_not_skipped", "if (pidx >= 0 && pidx < P && (!live || live[l * P + pidx])) {", "if (pidx >= 0 && pidx < P) {", 0),
    ("candidates_threshold_strict", "match_idx[lq] = (bi >= 0 && bs >= tau) ? bi : -1;", "match_idx[lq] = (bi >= 0 && bs > tau) ? bi : -1;", 0),
    ("layer_mean_divisor_with_head_dim", "S[q * P + p] += (sqrt(sk) + sqrt(sv)) / (2.0 * T * H);", "S[q * P + p] += (sqrt(sk) + sqrt(sv)) / (2.0 * T * H * Dh);", 0),
    ("layer_mean_joint_root", "S[q * P + p] += (sqrt(sk) + sqrt(sv)) / (2.0 * T * H);", "S[q * P + p] += sqrt(sk + sv) / (2.0 * T * H);", 0),
    ("layer_mean_squared_distance", "S[q * P + p] += (sqrt(sk) + sqrt(sv)) / (2.0 * T * H);", "S[q * P + p] += (sk + sv) / (2.0 * T * H);", 0),
    ("layer_mean_sum_not_mean", "const double d = S[q * P + p] / L;", "const double d = S[q * P + p];", 0),
    ("layer_mean_v_dropped", "          sv += b * b;\n        }\n        S[q * P + p]", "          sv += 0.0 * b;\n        }\n        S[q * P + p]", 0),
    ("layer_mean_dead_not_skipped", "if (live && !live[p]) continue;", "", 0),
    ("layer_mean_tie_highest_index", "if (d < bd) { sd = bd; bd = d; bi = (int32_t)p; }", "if (d <= bd) { sd = bd; bd = d; bi = (int32_t)p; }", 0),
    ("layer_mean_runner_up_not_demoted", "if (d < bd) { sd = bd; bd = d; bi = (int32_t)p; }", "if (d < bd) { bd = d; bi = (int32_t)p; }", 0),
    ("layer_mean_threshold_strict", "match_idx[q] = (bi >= 0 && bd <= thr) ? bi : -1;\n  }\ndone:", "match_idx[q] = (bi >= 0 && bd < thr) ? bi : -1;\n  }\ndone:", 0),
    ("cand_dist_divisor", "sum += (sqrt(sk) + sqrt(sv)) / (2.0 * T * H);", "sum += (sqrt(sk) + sqrt(sv)) / (2.0 * T);", 0),
    ("cand_dist_sum_not_mean", "d = sum / L;", "d = sum;", 0),
    ("cand_dist_k_against_v", "const double a = buf[i] - buf[2 * D + i], b = buf[D + i] - buf[3 * D + i];", "const double a = buf[i] - buf[3 * D + i], b = buf[D + i] - buf[2 * D + i];", 0),
    ("cand_dist_tie_highest_index", "if (d < bd || (d == bd && pidx < bi)) { bd = d; bi = pidx; }", "if (d <= bd) { bd = d; bi = pidx; }", 0),
    ("cand_dist_dead_not_skipped", "if (pidx >= 0 && pidx < P && (!live || live[pidx])) {", "if (pidx >= 0 && pidx < P) {", 0),
    ("cand_dist_threshold_strict", "match_idx[q] = (bi >= 0 && bd <= thr) ? bi : -1;\n    free(buf);", "match_idx[q] = (bi >= 0 && bd < thr) ? bi : -1;\n    free(buf);", 0),
    ("pat_rank_floor", "int64_t k = (int64_t)ceil(p * (double)m / 100.0);", "int64_t k = (int64_t)floor(p * (double)m / 100.0);", 0),
    ("pat_rank_off_by_one", "*threshold = s[k - 1];", "*threshold = s[k < m ? k : m - 1];", 0),
    ("pat_nonfinite_kept", "if (isfinite(samples[i])) s[m++] = samples[i];", "if (!isnan(samples[i])) s[m++] = samples[i];", 0),
    ("pat_fraction_not_percent", "ceil(p * (double)m / 100.0)", "ceil(p * (double)m)", 0),
    ("apply_threshold_strict", "(best_idx[i] >= 0 && best_dist[i] <= thr) ? best_idx[i] : -1;", "(best_idx[i] >= 0 && best_dist[i] < thr) ? best_idx[i] : -1;", 0),
    ("admit_matched_also_admitted", "if (match_idx[q] >= 0) continue;", "if (match_idx[q] > 0) continue;", 0),
    ("admit_slot_not_marked_live", "    live[s] = 1;\n", "", 0),
    ("admit_norms_swapped", "p_vsq[((int64_t)l * P + s) * nh + h] = q_vsq[((int64_t)l * Q + q) * nh + h];", "p_vsq[((int64_t)l * P + s) * nh + h] = q_ksq[((int64_t)l * Q + q) * nh + h];", 0),
    ("admit_v_not_copied", "memcpy(vp + (int64_t)l * p_layer_stride + s * block_elems, vq +", "memcpy(vp + (int64_t)l * p_layer_stride + s * block_elems, kq +", 0),
    ("admit_highest_free_slot", "while (next < P && live[next]) ++next;\n    if (next >= P) continue; /* pool full */\n    const int64_t s = next;",
     "while (next < P && live[P - 1 - next]) ++next;\n    if (next >= P) continue; /* pool full */\n    const int64_t s = P - 1 - next;", 0),
    ("remap_pool_ids_ignored", "redirect[query_ids[q]] = pool_ids ? pool_ids[m[q]] : m[q];", "redirect[query_ids[q]] = m[q];", 0),
    ("remap_target_gains_one", "refcount_out[(int64_t)l * NB + tgt] += (int32_t)cnt[b];", "refcount_out[(int64_t)l * NB + tgt] += 1;", 0),
    ("remap_query_keeps_references", "refcount_out[(int64_t)l * NB + b] -= (int32_t)cnt[b];", "", 0),
    ("remap_freed_flag_early", "(refcount_out[(int64_t)l * NB + query_ids[q]] == 0);", "(refcount_out[(int64_t)l * NB + query_ids[q]] <= 1);", 0),
    ("remap_padding_redirected", "if (b >= 0 && b < NB) {\n        cnt[b] += 1;", "if (b >= -1 && b < NB) { if (b < 0) b = 0;\n        cnt[b] += 1;", 0),
    ("remap_counts_entries_not_changes", "if (redirect[b] != b) changed += 1;", "changed += 1;", 0),
    ("remap_layers_share_matches", "const int32_t* m = match_idx + (int64_t)l * Q;", "const int32_t* m = match_idx;", 0),
]


def make_mutant(src, old, new, which):
    n = src.count(old)
    assert n > 0, f"mutant text not found in the oracle source: {old!r}"
    if which is None:
        return src.replace(old, new)
    assert which < n, f"occurrence {which} of {n}"
    pos = -1
    for _ in range(which + 1):
        pos = src.index(old, pos + 1)
    return src[:pos] + new + src[pos + len(old):]


BY_NAME = {m[0]: m for m in MUTANTS}


def build_mutant(workdir, name):
    """Compile mutant `name` into workdir/name/libmutant.so and return that path."""
    _, old, new, which = BY_NAME[name]
    src = open(SRC).read()
    mutated = make_mutant(src, old, new, which)
    assert mutated != src
    d = os.path.join(workdir, name)
    os.makedirs(d, exist_ok=True)
    c, lib = os.path.join(d, "mutant.c"), os.path.join(d, "libmutant.so")
    with open(c, "w") as f:
        f.write(mutated)
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-w", "-o", lib, c, "-lm"])
    return lib
