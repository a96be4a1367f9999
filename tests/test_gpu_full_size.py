"""Parity at the full sizes of the benchmark workloads, in the launch configuration bench.py times.

The oracle cannot score a whole workload in reasonable time, so each test combines
  (1) every query of every layer: the score the GPU reports must be the oracle's score of the
      block the GPU picked (one from-scratch pair score per query),
  (2) properties that follow from how the inputs were planted (which queries must match what),
  (3) the first, a middle and the last layer, 128 queries each: the full oracle search over the whole pool,
      compared by the ambiguity rule (bit-exact index and decision outside the reported near-ties),
  (4) the remap on all layers against the oracle remap fed with the GPU's decisions (bit-exact).
Needs a real MI355X and its 288 GB.
"""
import sys

import numpy as np
import pytest
import torch

from paper_2507_21433_amd import binding as rc
from paper_2507_21433_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def dcode(w):
    return 0 if w.dtype == "f16" else 1


@pytest.fixture(autouse=True)
def _free_cached_hbm():
    torch.cuda.empty_cache()
    yield
    torch.cuda.empty_cache()


def run_path(w, pr):
    """norms -> match -> remap exactly as bench.py's step does (pool norms computed once)."""
    pk, pv = rc.rc_block_norms(pr["kp"], pr["vp"], w.mode)
    qk, qv = rc.rc_block_norms(pr["kq"], pr["vq"], w.mode)
    m = rc.rc_match_blocks(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, pr["live"], w.tau, w.mode)
    r = rc.rc_remap_block_table(pr["tables"], pr["query_ids"], None, m["match_idx"], w.P, w.NB, pr["refcount"])
    torch.cuda.synchronize()
    return ({k: v.cpu().numpy() for k, v in m.items()}, {k: v.cpu().numpy() for k, v in r.items()},
            (qk, qv, pk, pv))


def check_reported_scores(oracle, w, pr, gpu, layers):
    """(1): |best_score - oracle score of (q, best_idx)| <= 2e-3 for every query of the listed layers."""
    worst = 0.0
    for l in layers:
        idx = gpu["best_idx"][l]
        ok = idx >= 0
        q = np.flatnonzero(ok).astype(np.int32)
        # only the blocks involved travel to the host
        kq, vq = pr["kq"][l:l + 1], pr["vq"][l:l + 1]
        sel = torch.as_tensor(idx[ok].astype(np.int64), device=DEV)
        kp, vp = pr["kp"][l:l + 1][:, sel], pr["vp"][l:l + 1][:, sel]
        s = oracle.score_pairs(dcode(w), w.mode, synth.bits(kq), synth.bits(vq), synth.bits(kp), synth.bits(vp),
                               np.zeros(q.size, np.int32), q, np.arange(q.size, dtype=np.int32))
        err = np.abs(gpu["best_score"][l][ok].astype(np.float64) - s)
        worst = max(worst, float(err.max()) if err.size else 0.0)
        assert err.size == 0 or err.max() <= parity.TOL, f"layer {l}: reported score off by {err.max():.3e}"
    return worst


def check_sampled_search(oracle, w, pr, gpu, layers, queries):
    """(3): full oracle search on the listed layers for a contiguous query range."""
    rep = []
    for l in layers:
        qs = slice(queries[0], queries[1])
        say(f"{w.name}: oracle search, layer {l}, queries {queries[0]}..{queries[1] - 1}")
        a = [synth.bits(pr[n][l:l + 1][:, qs]) if n[1] == "q" else synth.bits(pr[n][l:l + 1]) for n in ("kq", "vq", "kp", "vp")]
        orc = oracle.match(dcode(w), w.mode, *a, pr["live"][l:l + 1].cpu().numpy(), w.tau, want_scores=True)
        g = {k: v[l:l + 1, qs] for k, v in gpu.items()}
        rep.append(parity.check_match(g, orc, w.tau, parity.score_lookup(orc["scores"], g["best_idx"])))
    return rep


def check_remap_all_layers(oracle, w, pr, gpu, remap):
    """(4): oracle remap with the GPU's decisions, every layer, bit-exact."""
    o = oracle.remap(pr["tables"].cpu().numpy(), pr["query_ids"].cpu().numpy(), None, gpu["match_idx"], w.P, w.NB,
                     pr["refcount"].cpu().numpy())
    for k in ("tables", "refcount", "freed", "n_remapped"):
        assert np.array_equal(remap[k], o[k]), k
    # tables only point at blocks that are still referenced
    for l in range(0, w.L, max(1, w.L // 4)):
        t = remap["tables"][l]
        t = t[t >= 0]
        assert (remap["refcount"][l][t] >= 1).all()


def brief(rep):
    return [{k: v for k, v in r.items() if k != "ambiguous_list"} for r in rep]


def expected_planted_matches(w, plan):
    want = np.full(w.Q, -1)
    live_target = plan.live[plan.planted_targets] == 1
    want[plan.planted_slots[live_target]] = plan.planted_targets[live_target]
    return want


def test_cfg2_full(oracle):
    w = synth.WORKLOADS[2]
    say(f"{w.name} full size: L={w.L} P={w.P} Q={w.Q}")
    pr = synth.make_problem(w, DEV)
    gpu, remap, _ = run_path(w, pr)
    plan = pr["plan"]
    # (2) sigma = 0.15 copies score ~0.989 and match their target; fresh queries (|score| ~ 0.03) match nothing
    want = expected_planted_matches(w, plan)
    assert (gpu["match_idx"] == want[None]).all()
    assert np.allclose(gpu["best_score"][:, plan.planted_slots], 1 / np.sqrt(1 + w.sigma ** 2), atol=4e-3)
    worst = check_reported_scores(oracle, w, pr, gpu, range(w.L))
    rep = check_sampled_search(oracle, w, pr, gpu, (0, 31, 63), (0, w.Q))
    say(f"{w.name}: worst reported-score error {worst:.2e}; sampled layers {rep}")
    check_remap_all_layers(oracle, w, pr, gpu, remap)
    assert int(remap["n_remapped"].sum()) == w.L * int((want >= 0).sum())


def test_cfg3_full(oracle):
    w = synth.WORKLOADS[3]
    say(f"{w.name} full size: L={w.L} P={w.P} Q={w.Q} bf16")
    pr = synth.make_problem(w, DEV)
    gpu, remap, _ = run_path(w, pr)
    worst = check_reported_scores(oracle, w, pr, gpu, range(w.L))
    rep = (check_sampled_search(oracle, w, pr, gpu, (0,), (0, 128)) + check_sampled_search(oracle, w, pr, gpu, (31,), (448, 576))
           + check_sampled_search(oracle, w, pr, gpu, (63,), (896, 1024)))
    say(f"{w.name}: worst reported-score error {worst:.2e}; sampled {brief(rep)}")
    assert sum(r["near_tie"] for r in rep) > 0          # near-ties are the point of this workload ...
    # ... and still a good share of the sampled queries has a clear winner, for which index and decision must be bit-exact
    clear = sum(r["n"] - r["ambiguous"] for r in rep)
    assert clear >= 0.3 * sum(r["n"] for r in rep), f"only {clear} of the sampled queries are outside the near-tie band"
    check_remap_all_layers(oracle, w, pr, gpu, remap)


def test_cfg5_full(oracle):
    w = synth.WORKLOADS[5]
    say(f"{w.name} full size: L={w.L} P={w.P} Q={w.Q} T={w.T} per-head")
    pr = synth.make_problem(w, DEV)
    gpu, remap, _ = run_path(w, pr)
    plan = pr["plan"]
    want = expected_planted_matches(w, plan)
    assert (gpu["match_idx"] == want[None]).all()      # untouched heads score exactly 1, noisy ones ~0.995
    worst = check_reported_scores(oracle, w, pr, gpu, (0, 7, 15, 23, 31))
    rep = (check_sampled_search(oracle, w, pr, gpu, (0,), (0, 128)) + check_sampled_search(oracle, w, pr, gpu, (16,), (192, 320))
           + check_sampled_search(oracle, w, pr, gpu, (31,), (384, 512)))
    say(f"{w.name}: worst reported-score error {worst:.2e}; sampled {brief(rep)}")
    assert sum(r["n"] - r["ambiguous"] for r in rep) >= 0.5 * sum(r["n"] for r in rep)
    check_remap_all_layers(oracle, w, pr, gpu, remap)


def test_cfg4_full(oracle):
    w = synth.WORKLOADS[4]
    free, total = torch.cuda.mem_get_info()
    need = w.L * (w.P + w.Q) * w.block_bytes + (24 << 30)
    # an MI355X has 288 GB: too little free memory means something else holds it, which is a failure, not a skip
    assert free >= need, f"needs {need >> 30} GiB of free HBM, {free >> 30} GiB available"
    say(f"{w.name} full size: L={w.L} P={w.P} Q={w.Q} ({need >> 30} GiB)")
    pr = synth.make_problem(w, DEV)
    gpu, remap, _ = run_path(w, pr)
    plan = pr["plan"]
    # (2) plants aimed at live blocks match them, plants aimed at dead blocks and fresh queries match nothing
    want = expected_planted_matches(w, plan)
    assert (gpu["match_idx"] == want[None]).all()
    dead_plants = plan.planted_slots[plan.live[plan.planted_targets] == 0]
    assert dead_plants.size > 0 and (gpu["best_score"][:, dead_plants] < 0.2).all()
    worst = check_reported_scores(oracle, w, pr, gpu, (0, 16, 32, 48, 63))
    rep = (check_sampled_search(oracle, w, pr, gpu, (0,), (0, 128)) + check_sampled_search(oracle, w, pr, gpu, (32,), (448, 576))
           + check_sampled_search(oracle, w, pr, gpu, (63,), (896, 1024)))
    say(f"{w.name}: worst reported-score error {worst:.2e}; sampled {brief(rep)}")
    assert sum(r["n"] - r["ambiguous"] for r in rep) >= 0.5 * sum(r["n"] for r in rep)
    check_remap_all_layers(oracle, w, pr, gpu, remap)
    # dead pool blocks are never a table target
    t = remap["tables"][5]
    assert (plan.live[t[t < w.P]] == 1).all()
