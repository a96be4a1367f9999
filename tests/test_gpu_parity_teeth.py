"""The GPU parity tests must have teeth too: when the oracle is wrong, they must say so.

A few copies of the oracle with one planted mistake each (tests/mutants.py; the mistake is in the
oracle, on the CPU, never in the HIP path) are put in the oracle's place, and the parity tests of
the entry point the mistake concerns run in a child process, one at a time.  The HIP path runs
unchanged and correctly in every one of them; the child must report a failed comparison.  Mistakes
that only move which of several equally good blocks is picked (ties) are left out: the parity rule
accepts those by design.
"""
import os
import subprocess
import sys

import pytest

from tests.mutants import ROOT, build_mutant

pytestmark = pytest.mark.gpu

# (mutant, test file, -k selection): small cases only, a few seconds each
CASES = [
    ("norm_not_squared", "test_gpu_parity.py", "test_norms"),
    ("match_v_uses_k_tensor", "test_gpu_parity.py", "test_cfg1_tiny"),
    ("pair_score_not_halved", "test_gpu_candidates.py", "test_candidates_small"),
    ("match_dead_blocks_not_skipped", "test_gpu_parity.py", "test_match_ragged_tiles"),
    ("match_runner_up_not_raised", "test_gpu_parity.py", "test_cfg1_tiny"),
    ("match_head_mean_not_min", "test_gpu_parity.py", "test_per_head_mode"),
    ("layer_mean_joint_root", "test_gpu_layer_mean.py", "test_layer_mean_small"),
    ("layer_mean_dead_not_skipped", "test_gpu_layer_mean.py", "test_layer_mean_duplicates_ties_dead"),
    ("cand_dist_sum_not_mean", "test_gpu_candidates.py", "test_candidate_distances_small"),
    ("pat_rank_floor", "test_gpu_pat.py", "test_pat_random"),
    ("admit_norms_swapped", "test_gpu_pool.py", "test_admit_random"),
    ("remap_target_gains_one", "test_gpu_parity.py", "test_remap_random"),
    ("remap_freed_flag_early", "test_gpu_parity.py", "test_remap_random"),
    ("bf16_shift", "test_gpu_parity.py", "test_norms"),
    ("norms_k_and_v_swapped", "test_gpu_parity.py", "test_norms"),
    ("norms_layer_stride_ignored", "test_gpu_parity.py", "test_norms"),
    ("norm_head_filter_inverted", "test_gpu_parity.py", "test_norms"),
    ("layout_head_innermost", "test_gpu_parity.py", "test_norms"),
    ("cosine_zero_norm_and", "test_gpu_parity.py", "test_match_degenerate_blocks"),
    ("match_layer_stride_ignored", "test_gpu_parity.py", "test_match_ragged_tiles"),
    ("match_query_layer_stride_ignored", "test_gpu_parity.py", "test_layer_stride_padding"),
    ("match_head_norm_index", "test_gpu_parity.py", "test_per_head_mode"),
    ("match_head_v_uses_k_norm", "test_gpu_parity.py", "test_per_head_mode"),
    ("candidates_dead_not_skipped", "test_gpu_candidates.py", "test_candidates_small"),
    ("cand_dist_dead_not_skipped", "test_gpu_candidates.py", "test_candidate_distances_small"),
    ("cand_dist_k_against_v", "test_gpu_candidates.py", "test_candidate_distances_small"),
    ("cand_dist_query_layer_ignored", "test_gpu_candidates.py", "test_candidate_distances_small"),
    ("layer_mean_sum_not_mean", "test_gpu_layer_mean.py", "test_layer_mean_small"),
    ("layer_mean_divisor_with_head_dim", "test_gpu_layer_mean.py", "test_layer_mean_small"),
    ("layer_mean_runner_up_not_demoted", "test_gpu_layer_mean.py", "test_layer_mean_small"),
    ("layer_mean_pool_layer_stride_ignored", "test_gpu_layer_mean.py", "test_layer_mean_small"),
    ("pat_nonfinite_kept", "test_gpu_pat.py", "test_pat_special_values"),
    ("pat_rank_off_by_one", "test_gpu_pat.py", "test_pat_random"),
    ("apply_threshold_strict", "test_gpu_pat.py", "test_apply_threshold"),
    ("admit_slot_not_marked_live", "test_gpu_pool.py", "test_admit_random"),
    ("admit_highest_free_slot", "test_gpu_pool.py", "test_admit_random"),
    ("admit_v_not_copied", "test_gpu_pool.py", "test_admit_random"),
    ("admit_layers_after_first_not_copied", "test_gpu_pool.py", "test_admit_random"),
    ("admit_matched_also_admitted", "test_gpu_pool.py", "test_admit_random"),
    ("remap_pool_ids_ignored", "test_gpu_parity.py", "test_remap_random"),
    ("remap_padding_redirected", "test_gpu_parity.py", "test_remap_random"),
    ("remap_counts_entries_not_changes", "test_gpu_parity.py", "test_remap_random"),
    ("remap_layers_share_matches", "test_gpu_parity.py", "test_remap_random"),
    ("remap_query_keeps_references", "test_gpu_parity.py", "test_remap_random"),
    ("remap_out_of_range_entry_clamped", "test_gpu_parity.py", "test_remap_random"),
]


@pytest.mark.parametrize("mutant,test_file,select", CASES, ids=[c[0] for c in CASES])
def test_gpu_parity_rejects_wrong_oracle(tmp_path, mutant, test_file, select):
    print(f"[gpu-case] wrong oracle '{mutant}' against {test_file} -k {select}", flush=True)
    lib = build_mutant(str(tmp_path), mutant)
    env = dict(os.environ, RC_ORACLE_LIB=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", test_file), "-m", "gpu", "-x", "-q",
                        "-k", select, "-p", "no:cacheprovider", "--timeout", "120", "--timeout-method", "thread"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    # 1 = a comparison failed (what must happen); 0 = the wrong oracle went unnoticed; else the run itself broke
    assert r.returncode == 1, f"{mutant}: exit code {r.returncode}\n{r.stdout[-1500:]}\n{r.stderr[-500:]}"
    assert "AssertionError" in r.stdout or "assert" in r.stdout, r.stdout[-1500:]
