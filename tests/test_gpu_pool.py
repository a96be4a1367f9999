"""Parity of rc_pool_admit (streaming pool maintenance) with the CPU oracle, bit-exact, and a multi-step run of the
whole loop (norms -> layer-mean search -> admit) in which blocks admitted in one step are found in later ones.
Needs a real MI355X."""
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


def rand_kv(gen, L, n, T, H, dtype):
    return torch.randn((L, n, T, H, 128), generator=gen, device=DEV, dtype=torch.float32).to(dtype)


def admit_both(oracle, kq, vq, kp, vp, live, match, mode=0):
    """Runs the GPU call and the oracle on copies of the same state; returns both results for comparison."""
    qk, qv = rc.rc_block_norms(kq, vq, mode)
    pk, pv = rc.rc_block_norms(kp, vp, mode) if kp.shape[1] else (torch.empty((kp.shape[0], 0) + ((kp.shape[3],) if mode else ()), device=DEV),) * 2
    g = dict(kp=kp.clone(), vp=vp.clone(), pk=pk.clone(), pv=pv.clone(), live=live.clone())
    out = rc.rc_pool_admit(kq, vq, qk, qv, g["kp"], g["vp"], g["pk"], g["pv"], g["live"], match, mode)
    torch.cuda.synchronize()
    o = dict(kp=synth.bits(kp).copy(), vp=synth.bits(vp).copy(), pk=pk.cpu().numpy().astype(np.float64),
             pv=pv.cpu().numpy().astype(np.float64), live=live.cpu().numpy().copy())
    slot, n = oracle.pool_admit(synth.bits(kq), synth.bits(vq), qk.cpu().numpy().astype(np.float64),
                                qv.cpu().numpy().astype(np.float64), o["kp"], o["vp"], o["pk"], o["pv"], o["live"],
                                match.cpu().numpy())
    assert np.array_equal(out["slot_of_query"].cpu().numpy(), slot)
    assert int(out["n_admitted"].cpu()[0]) == n
    assert np.array_equal(g["live"].cpu().numpy(), o["live"])
    assert np.array_equal(synth.bits(g["kp"]), o["kp"]) and np.array_equal(synth.bits(g["vp"]), o["vp"])
    assert np.array_equal(g["pk"].cpu().numpy().astype(np.float64), o["pk"])
    assert np.array_equal(g["pv"].cpu().numpy().astype(np.float64), o["pv"])
    return g, slot, n


@pytest.mark.parametrize("L,P,Q,T,H,mode,dtype,dead_frac,match_frac", [
    (2, 300, 40, 16, 8, 0, torch.float16, 0.2, 0.3),
    (1, 10000, 1500, 16, 1, 0, torch.bfloat16, 0.1, 0.2),     # several chunks, more than 1024 queries
    (3, 5, 9, 32, 2, 1, torch.float16, 0.6, 0.0),             # more unmatched queries than free slots, per-head norms
    (2, 4097, 33, 16, 1, 0, torch.float16, 1.0, 0.5),         # an empty pool: every slot free
    (2, 64, 16, 16, 4, 0, torch.float16, 0.0, 0.0),           # a full pool
    (2, 64, 16, 16, 4, 1, torch.bfloat16, 0.5, 1.0),          # every query matched
])
def test_admit_random(oracle, L, P, Q, T, H, mode, dtype, dead_frac, match_frac):
    say(f"admit L={L} P={P} Q={Q} T={T} H={H} mode={mode} dead={dead_frac} matched={match_frac}")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(P * 31 + Q)
    kq, vq, kp, vp = (rand_kv(gen, L, n, T, H, dtype) for n in (Q, Q, P, P))
    rng = np.random.RandomState(Q)
    live = torch.as_tensor((rng.rand(P) >= dead_frac).astype(np.uint8), device=DEV)
    match = torch.as_tensor(np.where(rng.rand(Q) < match_frac, rng.randint(0, P, Q), -1).astype(np.int32), device=DEV)
    g, slot, n = admit_both(oracle, kq, vq, kp, vp, live, match, mode)
    n_free, n_unmatched = int((live == 0).sum()), int((match < 0).sum())
    assert n == min(n_free, n_unmatched)
    say(f"  admitted {n} of {n_unmatched} unmatched into {n_free} free slots")


def test_admit_empty_shapes_and_errors():
    say("admit: Q = 0, P = 0, bad workspace")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(1)
    kq, vq, kp, vp = (rand_kv(gen, 2, n, 16, 2, torch.float16) for n in (4, 4, 8, 8))
    qk, qv = rc.rc_block_norms(kq, vq, 0)
    pk, pv = rc.rc_block_norms(kp, vp, 0)
    live = torch.zeros(8, dtype=torch.uint8, device=DEV)
    m = torch.full((4,), -1, dtype=torch.int32, device=DEV)
    out = rc.rc_pool_admit(kq[:, :0].contiguous(), vq[:, :0].contiguous(), qk[:, :0].contiguous(), qv[:, :0].contiguous(),
                           kp, vp, pk, pv, live, m[:0].contiguous())
    torch.cuda.synchronize()
    assert int(out["n_admitted"][0]) == 0 and int(live.sum()) == 0
    out = rc.rc_pool_admit(kq, vq, qk, qv, kp[:, :0].contiguous(), vp[:, :0].contiguous(), pk[:, :0].contiguous(),
                           pv[:, :0].contiguous(), live[:0].contiguous(), m)
    torch.cuda.synchronize()
    assert int(out["n_admitted"][0]) == 0 and (out["slot_of_query"] == -1).all()
    with pytest.raises(rc.RcError) as e:
        rc.rc_pool_admit(kq, vq, qk, qv, kp, vp, pk, pv, live, m, workspace=torch.empty(16, dtype=torch.uint8, device=DEV))
    assert e.value.code == 3


def test_streaming_steps(oracle):
    # five decoding steps over one pool: 40 % of each step's new blocks are noisy copies of blocks that are live at
    # that moment (the ones admitted in earlier steps included); the rest find no partner and are admitted
    L, P, Q, T, H = 2, 400, 48, 16, 8
    say(f"streaming: 5 steps, L={L} P={P} Q={Q}")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(99)
    rng = np.random.RandomState(99)
    kp, vp = rand_kv(gen, L, P, T, H, torch.float16), rand_kv(gen, L, P, T, H, torch.float16)
    live = torch.ones(P, dtype=torch.uint8, device=DEV)
    live[250:] = 0                                                  # 150 free slots
    pk, pv = rc.rc_block_norms(kp, vp, 0)
    thr, tol = 0.5, parity.dist_tol(T, H, 128)
    admitted_so_far, hits_on_admitted = set(), 0
    for step in range(5):
        kq, vq = rand_kv(gen, L, Q, T, H, torch.float16), rand_kv(gen, L, Q, T, H, torch.float16)
        live_ids = np.flatnonzero(live.cpu().numpy())
        copies = rng.choice(Q, int(0.4 * Q), replace=False)
        prefer = sorted(admitted_so_far)[: len(copies) // 2]         # aim half of the copies at earlier admissions
        targets = np.array(prefer + list(rng.choice(live_ids, len(copies) - len(prefer), replace=False)))
        for q, t in zip(copies, targets):
            kq[:, q] = (kp[:, t].float() + 0.1 * torch.randn(kp[:, t].shape, generator=gen, device=DEV)).half()
            vq[:, q] = (vp[:, t].float() + 0.1 * torch.randn(vp[:, t].shape, generator=gen, device=DEV)).half()
        qk, qv = rc.rc_block_norms(kq, vq, 0)
        g = rc.rc_match_blocks_layer_mean(kq, vq, qk, qv, kp, vp, pk, pv, live, thr)
        torch.cuda.synchronize()
        gn = {k: v.cpu().numpy() for k, v in g.items()}
        # the decisions against the oracle's search on the same state
        o = oracle.layer_mean(0, synth.bits(kq), synth.bits(vq), synth.bits(kp), synth.bits(vp), live.cpu().numpy(), thr,
                              want_dist=True)
        rep = parity.check_layer_mean(gn, o, thr, parity.dist_lookup(o["dist"], gn["best_idx"]), 0.05 * tol)
        want = np.full(Q, -1)
        want[copies] = targets
        assert np.array_equal(gn["match_idx"], want)
        hits_on_admitted += len(set(gn["match_idx"][gn["match_idx"] >= 0].tolist()) & admitted_so_far)
        # the admission against the oracle's, fed with the same decisions, on copies of the same state
        ok, ov = synth.bits(kp).copy(), synth.bits(vp).copy()
        opk, opv = pk.cpu().numpy().astype(np.float64), pv.cpu().numpy().astype(np.float64)
        olive = live.cpu().numpy().copy()
        slot, n = oracle.pool_admit(synth.bits(kq), synth.bits(vq), qk.cpu().numpy().astype(np.float64),
                                    qv.cpu().numpy().astype(np.float64), ok, ov, opk, opv, olive, gn["match_idx"])
        out = rc.rc_pool_admit(kq, vq, qk, qv, kp, vp, pk, pv, live, g["match_idx"])
        torch.cuda.synchronize()
        assert np.array_equal(out["slot_of_query"].cpu().numpy(), slot) and int(out["n_admitted"][0]) == n
        assert np.array_equal(live.cpu().numpy(), olive)
        assert np.array_equal(synth.bits(kp), ok) and np.array_equal(synth.bits(vp), ov)
        assert np.array_equal(pk.cpu().numpy().astype(np.float64), opk)
        # the norm cache stays what a fresh reduction over the pool gives
        fk, fv = rc.rc_block_norms(kp, vp, 0)
        lv = live.bool()
        assert torch.equal(fk[:, lv], pk[:, lv]) and torch.equal(fv[:, lv], pv[:, lv])
        admitted_so_far |= set(slot[slot >= 0].tolist())
        say(f"  step {step}: {rep['matched']} matched, {n} admitted, {int(live.sum())} live")
    assert hits_on_admitted > 0
    assert int(live.sum()) == 250 + len(admitted_so_far)
