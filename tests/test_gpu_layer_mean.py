"""Parity of rc_match_blocks_layer_mean (the paper's layer-mean Euclidean block distance and the one decision per
block that follows from it) with the CPU oracle.  Needs a real MI355X."""
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


def gpu_layer_mean(pr, live, thr):
    qk, qv = rc.rc_block_norms(pr["kq"], pr["vq"], 0)
    pk, pv = rc.rc_block_norms(pr["kp"], pr["vp"], 0)
    out = rc.rc_match_blocks_layer_mean(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, live, thr)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


def shared_live(pr):
    """One flag per pool block for all layers: live where every layer says so."""
    return pr["live"].min(dim=0).values.contiguous()


def run_case(oracle, w, thr, live="plan", tweak=None, tol_scale=0.05):
    """tol_scale: fraction of the distance tolerance used for the comparison.  The full tolerance is only needed
    by (near-)duplicate pairs, where the square root magnifies the rounding of the radicand; noisy copies and
    fresh blocks agree to a few 1e-6, and the tighter bar keeps the index check sharp."""
    pr = synth.make_problem(w, DEV)
    if tweak:
        tweak(pr)
    lv = shared_live(pr) if live == "plan" else live
    gpu = gpu_layer_mean(pr, lv, thr)
    orc = oracle.layer_mean(dcode(w), *(synth.bits(pr[n]) for n in ("kq", "vq", "kp", "vp")),
                            None if lv is None else lv.cpu().numpy(), thr, want_dist=True)
    tol = tol_scale * parity.dist_tol(w.T, w.H, w.Dh)
    rep = parity.check_layer_mean(gpu, orc, thr, parity.dist_lookup(orc["dist"], gpu["best_idx"]), tol)
    say(f"{w.name}: {rep}")
    return pr, gpu, orc, rep


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("L,P,Q,T,H", [(3, 300, 40, 16, 8), (1, 513, 257, 16, 8), (4, 130, 5, 32, 8), (2, 257, 1, 16, 3),
                                       (7, 96, 300, 16, 1)])
def test_layer_mean_small(oracle, dtype, L, P, Q, T, H):
    w = synth.scaled(synth.WORKLOADS[2], name=f"lm_{dtype}_L{L}_P{P}_Q{Q}_T{T}_H{H}", L=L, P=P, Q=Q, T=T, H=H,
                     dtype=dtype, planted_frac=0.2, R=1, E=P + Q, seed=41)
    say(w.name)
    thr = 0.5 * np.sqrt(w.Dh / (w.T * w.H))      # copies sit at 0.15 units, fresh blocks at 1.41
    pr, gpu, orc, rep = run_case(oracle, w, thr)
    plan = pr["plan"]
    lv = shared_live(pr).cpu().numpy()
    ok = lv[plan.planted_targets] == 1
    assert (gpu["match_idx"][plan.planted_slots[ok]] == plan.planted_targets[ok]).all()
    fresh = np.setdiff1d(np.arange(w.Q), plan.planted_slots)
    assert (gpu["match_idx"][fresh] == -1).all()


def test_layer_mean_layer_groups(oracle):
    # enough tiles that a workgroup walks several layers: 5 layers in groups of 2, 2 and 1
    w = synth.scaled(synth.WORKLOADS[2], name="lm_groups", L=5, P=44000, Q=8, T=16, H=1, planted_frac=0.5, R=1,
                     E=44008, seed=43)
    say(f"{w.name}: L={w.L} P={w.P} Q={w.Q}")
    thr = 0.5 * np.sqrt(w.Dh / (w.T * w.H))
    pr, gpu, orc, rep = run_case(oracle, w, thr)
    plan = pr["plan"]
    lv = shared_live(pr).cpu().numpy()
    ok = lv[plan.planted_targets] == 1
    assert (gpu["match_idx"][plan.planted_slots[ok]] == plan.planted_targets[ok]).all()


def test_layer_mean_duplicates_ties_dead(oracle):
    w = synth.scaled(synth.WORKLOADS[2], name="lm_dups", L=3, P=200, Q=16, planted_frac=0.5, R=1, E=216, seed=47)
    say(w.name)

    def tweak(pr):
        # query 0 is an exact copy of pool block 7 in every layer; pool blocks 150 and 20 are copies of block 7 too
        for n in ("k", "v"):
            pr[n + "q"][:, 0] = pr[n + "p"][:, 7]
            pr[n + "p"][:, 150] = pr[n + "p"][:, 7]
            pr[n + "p"][:, 20] = pr[n + "p"][:, 7]
            pr[n + "q"][:, 1] = 0                       # an all-zero query block
            pr[n + "q"][:, 2] = pr[n + "p"][:, 33]      # the only copy of block 33, which is dead
    live = torch.ones(w.P, dtype=torch.uint8, device=DEV)
    live[7] = 0                                         # the original is dead: the lowest live copy (20) must win
    live[33] = 0                                        # dead blocks are skipped by the search, not rejected after it
    pr, gpu, orc, rep = run_case(oracle, w, 0.5, live=live, tweak=tweak, tol_scale=1.0)
    tol = parity.dist_tol(w.T, w.H, w.Dh)
    assert orc["best_dist"][0] == 0.0 and gpu["best_dist"][0] <= tol and gpu["best_idx"][0] in (20, 150)
    assert gpu["match_idx"][0] == gpu["best_idx"][0]
    assert abs(gpu["second_dist"][0] - gpu["best_dist"][0]) <= tol       # the other copy is the runner-up
    # identical pool blocks see the same instruction sequence, so their distances are bit-identical and the lowest wins
    assert gpu["best_idx"][0] == 20
    assert np.isfinite(gpu["best_dist"]).all() and (gpu["best_dist"] >= 0).all()
    assert gpu["best_idx"][2] not in (-1, 33) and gpu["best_dist"][2] > 0.5 and gpu["match_idx"][2] == -1


def test_layer_mean_empty_and_errors():
    say("layer mean: no live block, P = 0, Q = 0, bad arguments")
    w = synth.scaled(synth.WORKLOADS[1], L=2, P=8, Q=4, E=8)
    pr = synth.make_problem(w, DEV)
    qk, qv = rc.rc_block_norms(pr["kq"], pr["vq"], 0)
    pk, pv = rc.rc_block_norms(pr["kp"], pr["vp"], 0)
    dead = torch.zeros(w.P, dtype=torch.uint8, device=DEV)
    out = rc.rc_match_blocks_layer_mean(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, dead, 1e9)
    torch.cuda.synchronize()
    assert (out["best_idx"] == -1).all() and (out["match_idx"] == -1).all()
    assert torch.isposinf(out["best_dist"]).all() and torch.isposinf(out["second_dist"]).all()
    kp0, vp0 = pr["kp"][:, :0].contiguous(), pr["vp"][:, :0].contiguous()
    out = rc.rc_match_blocks_layer_mean(pr["kq"], pr["vq"], qk, qv, kp0, vp0, pk[:, :0].contiguous(),
                                        pv[:, :0].contiguous(), None, 1e9)
    torch.cuda.synchronize()
    assert (out["best_idx"] == -1).all() and torch.isposinf(out["best_dist"]).all()
    kq0, vq0 = pr["kq"][:, :0].contiguous(), pr["vq"][:, :0].contiguous()
    out = rc.rc_match_blocks_layer_mean(kq0, vq0, qk[:, :0].contiguous(), qv[:, :0].contiguous(), pr["kp"], pr["vp"],
                                        pk, pv, None, 1.0)
    assert out["best_idx"].numel() == 0
    with pytest.raises(rc.RcError) as e:   # workspace too small
        rc.rc_match_blocks_layer_mean(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, None, 1.0,
                                      workspace=torch.empty(16, dtype=torch.uint8, device=DEV))
    assert e.value.code == 3
    with pytest.raises(rc.RcError) as e:   # NaN threshold
        rc.rc_match_blocks_layer_mean(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, None, float("nan"))
    assert e.value.code == 1


def full_size_case(oracle, w, n_samples=6):
    pr = synth.make_problem(w, DEV)
    plan = pr["plan"]
    lv = shared_live(pr)
    thr = 0.5
    gpu = gpu_layer_mean(pr, lv, thr)
    want = np.full(w.Q, -1)
    ok = lv.cpu().numpy()[plan.planted_targets] == 1
    want[plan.planted_slots[ok]] = plan.planted_targets[ok]
    assert (gpu["match_idx"] == want).all()
    assert np.allclose(gpu["best_dist"][plan.planted_slots[ok]], w.sigma, rtol=0.02)     # sigma * sqrt(Dh/(T H)) = sigma
    fresh = np.setdiff1d(np.arange(w.Q), plan.planted_slots)
    assert np.allclose(gpu["best_dist"][fresh], np.sqrt(2), rtol=0.02)
    # oracle over all layers on a sub-pool: per sampled query the GPU's pick, then 22 random live blocks
    rng = np.random.RandomState(2)
    qs = np.concatenate([plan.planted_slots[:n_samples], fresh[:n_samples]])
    tol = parity.dist_tol(w.T, w.H, w.Dh)
    worst = 0.0
    live_ids = np.flatnonzero(lv.cpu().numpy())
    for q in qs:
        sub = np.unique(np.concatenate([[gpu["best_idx"][q]], rng.choice(live_ids, 22, replace=False)]))
        sel = torch.as_tensor(sub, device=DEV)
        a = [synth.bits(pr[n][:, q:q + 1]) for n in ("kq", "vq")] + [synth.bits(pr[n][:, sel]) for n in ("kp", "vp")]
        o = oracle.layer_mean(dcode(w), *a, None, thr, want_dist=True)
        at = int(np.flatnonzero(sub == gpu["best_idx"][q])[0])
        err = abs(o["dist"][0, at] - float(gpu["best_dist"][q]))
        worst = max(worst, err)
        assert err <= tol, f"query {q}: distance off by {err:.3e}"
        assert o["dist"][0].min() >= o["dist"][0, at] - tol        # nothing in the sample beats the GPU's pick
    say(f"{w.name}: worst sampled distance error {worst:.2e}")


def test_layer_mean_cfg2_full(oracle):
    # the QwQ-32B-shaped step, all 64 layers folded into one decision per block (one layer per workgroup)
    w = synth.WORKLOADS[2]
    say(f"layer mean on {w.name}: L={w.L} P={w.P} Q={w.Q}")
    full_size_case(oracle, w)


def test_layer_mean_cfg4_full(oracle):
    # the 210 GB pool: every workgroup walks all 64 layers of its tile
    w = synth.WORKLOADS[4]
    torch.cuda.empty_cache()
    free, total = torch.cuda.mem_get_info()
    need = w.L * (w.P + w.Q) * w.block_bytes + (24 << 30)
    if free < need:
        pytest.skip(f"needs {need >> 30} GiB of free HBM, {free >> 30} GiB available")
    say(f"layer mean on {w.name}: L={w.L} P={w.P} Q={w.Q} ({need >> 30} GiB)")
    full_size_case(oracle, w, n_samples=4)
    torch.cuda.empty_cache()
