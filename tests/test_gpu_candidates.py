"""Parity of rc_score_candidates (candidate-restricted Stage 2) with the CPU oracle.  Needs a real MI355X."""
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


def gpu_candidates(w, pr, cand, live):
    qk, qv = rc.rc_block_norms(pr["kq"], pr["vq"], w.mode)
    pk, pv = rc.rc_block_norms(pr["kp"], pr["vp"], w.mode)
    out = rc.rc_score_candidates(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, live,
                                 torch.as_tensor(cand, device=DEV), w.tau, w.mode)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


AMB = 2e-5   # fp32 accumulation over 16K..64K exact products: observed error 3e-7, bound ~1e-5


def compare(gpu, orc, cand, tau, tol=parity.TOL, amb=AMB):
    """Scores to tol everywhere; the pick bit-exact unless another candidate is within amb of the best or of tau."""
    gs, os_ = gpu["scores"].astype(np.float64), orc["scores"]
    fin = np.isfinite(os_)
    assert np.array_equal(np.isfinite(gs), fin), "validity of candidates differs"
    assert (gs[~fin] == -np.inf).all()
    err = np.abs(gs[fin] - os_[fin]).max() if fin.any() else 0.0
    assert err <= tol, f"candidate score off by {err:.3e}"
    best = orc["best_score"]
    # runner-up among candidates that name a different pool block than the best
    other = np.where((cand != orc["best_idx"][..., None]) & fin, os_, -np.inf).max(axis=-1) if cand.shape[-1] else np.full(best.shape, -np.inf)
    with np.errstate(invalid="ignore"):          # -inf - -inf for a list without a valid entry
        amb = (best - other <= amb) | (np.abs(best - tau) <= amb)
    clear = ~amb
    assert np.array_equal(gpu["best_idx"][clear], orc["best_idx"][clear])
    assert np.array_equal(gpu["match_idx"][clear], orc["match_idx"][clear])
    has = orc["best_idx"] >= 0
    assert np.array_equal(gpu["best_idx"] >= 0, has)
    assert np.abs(gpu["best_score"][has].astype(np.float64) - best[has]).max(initial=0.0) <= tol
    return dict(max_score_err=float(err), ambiguous=int((amb & has).sum()), lists=int(has.sum()))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("mode,T,H", [(0, 16, 8), (1, 16, 8), (1, 32, 8), (0, 16, 3), (1, 16, 4), (0, 32, 16),
                                      (1, 16, 3), (1, 32, 10), (1, 16, 5), (1, 16, 16), (1, 32, 1)])  # head counts that do not divide 16 too
def test_candidates_small(oracle, dtype, mode, T, H):
    w = synth.scaled(synth.WORKLOADS[2], name=f"cand_{dtype}_m{mode}_T{T}_H{H}", L=2, P=300, Q=40, T=T, H=H, mode=mode,
                     dtype=dtype, planted_frac=0.3, R=1, E=340, seed=31)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    plan = pr["plan"]
    rng = np.random.RandomState(3)
    C = 7
    cand = rng.randint(0, w.P, size=(w.L, w.Q, C)).astype(np.int32)
    cand[:, plan.planted_slots, 2] = plan.planted_targets[None]       # the true partner is in the list
    cand[:, :, 5] = -1                                                 # empty slot
    cand[0, 0, 0] = w.P + 5                                            # out of range
    cand[:, 3, 1] = cand[:, 3, 4]                                      # the same block listed twice
    cand[1, 7, :] = -1                                                 # an empty list
    live = pr["live"].clone()
    live[0, int(plan.planted_targets[0])] = 0                          # a true partner is dead in layer 0
    gpu = gpu_candidates(w, pr, cand, live)
    orc = oracle.candidates(dcode(w), w.mode, *(synth.bits(pr[n]) for n in ("kq", "vq", "kp", "vp")), cand,
                            live.cpu().numpy(), w.tau)
    rep = compare(gpu, orc, cand, w.tau)
    say(f"{w.name}: {rep}")
    assert gpu["best_idx"][1, 7] == -1 and gpu["match_idx"][1, 7] == -1 and np.isneginf(gpu["best_score"][1, 7])
    slots = plan.planted_slots[plan.planted_slots != 7]
    assert (gpu["match_idx"][1, slots] == plan.planted_targets[plan.planted_slots != 7]).all()


def test_candidates_empty_and_errors():
    say("candidates: C = 0 and argument errors")
    w = synth.scaled(synth.WORKLOADS[1], P=8, Q=4, E=8)
    pr = synth.make_problem(w, DEV)
    qk, qv = rc.rc_block_norms(pr["kq"], pr["vq"], 0)
    pk, pv = rc.rc_block_norms(pr["kp"], pr["vp"], 0)
    cand = torch.empty((w.L, w.Q, 0), dtype=torch.int32, device=DEV)
    out = rc.rc_score_candidates(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, None, cand, 0.5, 0)
    torch.cuda.synchronize()
    assert (out["best_idx"] == -1).all() and (out["match_idx"] == -1).all() and torch.isneginf(out["best_score"]).all()


def test_candidates_cfg2_full(oracle):
    # the QwQ-32B-shaped step with 16 candidates per query, the planted partner among them
    w = synth.WORKLOADS[2]
    say(f"candidates on {w.name}: L={w.L} Q={w.Q} C=16")
    pr = synth.make_problem(w, DEV)
    plan = pr["plan"]
    rng = np.random.RandomState(9)
    C = 16
    cand = rng.randint(0, w.P, size=(w.L, w.Q, C)).astype(np.int32)
    cand[:, plan.planted_slots, 11] = plan.planted_targets[None]
    gpu = gpu_candidates(w, pr, cand, pr["live"])
    want = np.full(w.Q, -1)
    want[plan.planted_slots] = plan.planted_targets
    assert (gpu["match_idx"] == want[None]).all()
    for l in (0, 40, 63):
        a = [synth.bits(pr[n][l:l + 1]) for n in ("kq", "vq", "kp", "vp")]
        orc = oracle.candidates(0, w.mode, *a, cand[l:l + 1], pr["live"][l:l + 1].cpu().numpy(), w.tau)
        g = {k: v[l:l + 1] for k, v in gpu.items()}
        rep = compare(g, orc, cand[l:l + 1], w.tau)
        say(f"layer {l}: {rep}")


# ---- layer-mean distance of listed pairs (Stage 2 as the paper runs it)

def compare_distances(gpu, orc, cand, thr, tol):
    gd, od = gpu["dist"].astype(np.float64), orc["dist"]
    fin = np.isfinite(od)
    assert np.array_equal(np.isfinite(gd), fin) and np.isposinf(gd[~fin]).all()
    err = np.abs(gd[fin] - od[fin]).max() if fin.any() else 0.0
    assert err <= tol, f"distance off by {err:.3e}"
    best = orc["best_dist"]
    other = np.where((cand != orc["best_idx"][:, None]) & fin, od, np.inf).min(axis=-1) if cand.shape[-1] else np.full(best.shape, np.inf)
    with np.errstate(invalid="ignore"):          # inf - inf for a list without a valid entry
        clear = ~((other - best <= tol) | (np.abs(best - thr) <= tol))
    assert np.array_equal(gpu["best_idx"][clear], orc["best_idx"][clear])
    assert np.array_equal(gpu["match_idx"][clear], orc["match_idx"][clear])
    has = orc["best_idx"] >= 0
    assert np.array_equal(gpu["best_idx"] >= 0, has) and np.isposinf(gpu["best_dist"][~has]).all()
    assert np.abs(gpu["best_dist"][has].astype(np.float64) - best[has]).max(initial=0.0) <= tol
    return dict(max_err=float(err), clear=int((clear & has).sum()), lists=int(has.sum()))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("L,T,H,C", [(3, 16, 8, 7), (5, 32, 8, 20), (1, 16, 3, 1), (7, 16, 1, 16)])
def test_candidate_distances_small(oracle, dtype, L, T, H, C):
    w = synth.scaled(synth.WORKLOADS[2], name=f"cd_{dtype}_L{L}_T{T}_H{H}_C{C}", L=L, P=300, Q=40, T=T, H=H, dtype=dtype,
                     planted_frac=0.3, R=1, E=340, seed=33)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    plan = pr["plan"]
    rng = np.random.RandomState(5)
    cand = rng.randint(0, w.P, size=(w.Q, C)).astype(np.int32)
    cand[plan.planted_slots, C // 2] = plan.planted_targets           # the true partner is in the list
    if C > 2:
        cand[:, 1] = -1                                               # empty slot
        cand[0, 0] = w.P + 5                                          # out of range
        cand[7, :] = -1                                               # an empty list
    live = pr["live"].min(dim=0).values.contiguous().clone()
    live[int(plan.planted_targets[0])] = 0                            # a true partner is dead
    unit = np.sqrt(w.Dh / (w.T * w.H))
    thr = 0.5 * unit
    out = rc.rc_candidate_distances(pr["kq"], pr["vq"], pr["kp"], pr["vp"], live, torch.as_tensor(cand, device=DEV), thr)
    torch.cuda.synchronize()
    gpu = {k: v.cpu().numpy() for k, v in out.items()}
    orc = oracle.candidate_distances(dcode(w), *(synth.bits(pr[n]) for n in ("kq", "vq", "kp", "vp")), cand,
                                     live.cpu().numpy(), thr)
    rep = compare_distances(gpu, orc, cand, thr, 1e-5 * unit)         # direct differences in fp32: no cancellation
    say(f"{w.name}: {rep}")
    ok = (live.cpu().numpy()[plan.planted_targets] == 1) & (plan.planted_slots != 7 if C > 2 else True)
    assert (gpu["match_idx"][plan.planted_slots[ok]] == plan.planted_targets[ok]).all()
    # exact copies sit at exactly 0 here (the exhaustive search's expansion would leave ~5e-4)
    for n in ("k", "v"):
        pr[n + "q"][:, 3] = pr[n + "p"][:, 11]
    cand[3, 0] = 11
    live[11] = 1
    out = rc.rc_candidate_distances(pr["kq"], pr["vq"], pr["kp"], pr["vp"], live, torch.as_tensor(cand, device=DEV), thr)
    torch.cuda.synchronize()
    assert float(out["dist"][3, 0]) == 0.0 and int(out["match_idx"][3]) == 11


def test_candidate_distances_empty_and_errors():
    say("candidate distances: C = 0, P = 0, bad workspace")
    w = synth.scaled(synth.WORKLOADS[1], L=2, P=8, Q=4, E=8)
    pr = synth.make_problem(w, DEV)
    out = rc.rc_candidate_distances(pr["kq"], pr["vq"], pr["kp"], pr["vp"], None,
                                    torch.empty((4, 0), dtype=torch.int32, device=DEV), 1.0)
    torch.cuda.synchronize()
    assert (out["best_idx"] == -1).all() and torch.isposinf(out["best_dist"]).all() and (out["match_idx"] == -1).all()
    out = rc.rc_candidate_distances(pr["kq"], pr["vq"], pr["kp"][:, :0].contiguous(), pr["vp"][:, :0].contiguous(), None,
                                    torch.zeros((4, 3), dtype=torch.int32, device=DEV), 1.0)
    torch.cuda.synchronize()
    assert (out["best_idx"] == -1).all() and torch.isposinf(out["dist"]).all()
    with pytest.raises(rc.RcError) as e:
        rc.rc_candidate_distances(pr["kq"], pr["vq"], pr["kp"], pr["vp"], None, torch.zeros((4, 64), dtype=torch.int32, device=DEV),
                                  1.0, workspace=torch.empty(16, dtype=torch.uint8, device=DEV))
    assert e.value.code == 3


def test_candidate_distances_cfg2_full(oracle):
    w = synth.WORKLOADS[2]
    say(f"candidate distances on {w.name}: L={w.L} Q={w.Q} C=16")
    pr = synth.make_problem(w, DEV)
    plan = pr["plan"]
    rng = np.random.RandomState(9)
    C = 16
    cand = rng.randint(0, w.P, size=(w.Q, C)).astype(np.int32)
    cand[plan.planted_slots, 11] = plan.planted_targets
    live = pr["live"].min(dim=0).values.contiguous()
    out = rc.rc_candidate_distances(pr["kq"], pr["vq"], pr["kp"], pr["vp"], live, torch.as_tensor(cand, device=DEV), 0.5)
    torch.cuda.synchronize()
    gpu = {k: v.cpu().numpy() for k, v in out.items()}
    want = np.full(w.Q, -1)
    ok = live.cpu().numpy()[plan.planted_targets] == 1
    want[plan.planted_slots[ok]] = plan.planted_targets[ok]
    assert (gpu["match_idx"] == want).all()
    # the oracle on 12 whole lists (all 64 layers)
    qs = np.concatenate([plan.planted_slots[:6], np.setdiff1d(np.arange(w.Q), plan.planted_slots)[:6]])
    sub = {n: synth.bits(pr[n][:, torch.as_tensor(qs, device=DEV)]) for n in ("kq", "vq")}
    orc = oracle.candidate_distances(0, sub["kq"], sub["vq"], synth.bits(pr["kp"]), synth.bits(pr["vp"]), cand[qs],
                                     live.cpu().numpy(), 0.5)
    g = {k: v[qs] for k, v in gpu.items()}
    say(f"{w.name}: {compare_distances(g, orc, cand[qs], 0.5, 1e-5)}")
