"""Parity of rc_pool_touch, rc_refcount_release and rc_pool_evict with the CPU oracle (bit-exact), and the
steady state of the streaming pool: decoding steps that go on after the pool has filled up, in which blocks of
ended requests lose their references, leave the pool in LRU order and make room for the new ones.  Needs a real
MI355X."""
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


def t(a):
    return torch.as_tensor(np.ascontiguousarray(a), device=DEV)


def test_touch_and_release(oracle):
    say("touch / release")
    rng = np.random.RandomState(5)
    for P, n in ((1, 1), (50, 7), (70000, 100000), (300, 0)):
        arr = rng.randint(0, 9, P).astype(np.int32)
        slots = rng.randint(-2, P + 2, n).astype(np.int32)
        g = rc.rc_pool_touch(t(slots), 1234, t(arr.copy())) if n else t(arr.copy())
        want = oracle.pool_touch(slots, 1234, arr.copy())
        refc = rng.randint(0, 5, P).astype(np.int32)
        ids = rng.randint(-2, P + 2, n).astype(np.int32)
        ids[: n // 3] = ids[0] if n else 0                  # one id listed many times
        g2 = rc.rc_refcount_release(t(ids), t(refc.copy())) if n else t(refc.copy())
        torch.cuda.synchronize()
        assert np.array_equal(g.cpu().numpy(), want)
        assert np.array_equal(g2.cpu().numpy(), oracle.refcount_release(ids, refc.copy()))


def evict_both(oracle, live, refc, used, match, extra):
    lv = t(live.copy())
    out = rc.rc_pool_evict(lv, None if refc is None else t(refc), t(used), t(match), extra)
    torch.cuda.synchronize()
    want = live.copy()
    n_free, n_ev = oracle.pool_evict(want, refc, used, match, extra)
    assert np.array_equal(lv.cpu().numpy(), want)
    assert (int(out["n_free"].item()), int(out["n_evicted"].item())) == (n_free, n_ev)
    return n_free, n_ev


def test_evict_random(oracle):
    rng = np.random.RandomState(77)
    for case in range(60):
        P = int(rng.choice([1, 2, 63, 64, 65, 1023, 1024, 1025, 5000, 49152]))
        live = (rng.rand(P) < rng.choice([0.5, 0.95, 1.0])).astype(np.uint8)
        refc = (rng.randint(0, 3, P) * (rng.rand(P) < rng.choice([0.2, 0.6, 1.0]))).astype(np.int32)
        span = int(rng.choice([1, 2, 7, 300, 2 ** 31 - 1]))
        used = rng.randint(0, span, P).astype(np.int32)
        if rng.rand() < 0.3:
            used -= span // 2                                   # negative stamps sort below positive ones
        Q = int(rng.choice([0, 1, 40, 1024, 3000]))
        match = np.where(rng.rand(Q) < rng.choice([0.0, 0.6, 1.0]), -1, 3).astype(np.int32)
        extra = int(rng.choice([0, 0, 5, 100000]))
        use_rc = rng.rand() < 0.7
        say(f"evict case {case}: P={P} Q={Q} unmatched={(match < 0).sum()} extra={extra} refcounts={use_rc} stamps<{span}")
        evict_both(oracle, live, refc if use_rc else None, used, match, extra)


def test_evict_edges(oracle):
    say("evict: empty pool, nothing wanted, everything referenced, all stamps equal")
    z = np.zeros(0, np.int32)
    assert evict_both(oracle, np.zeros(0, np.uint8), None, z, np.array([-1, -1], np.int32), 0) == (0, 0)
    live = np.ones(3000, np.uint8)
    used = np.full(3000, 4, np.int32)
    assert evict_both(oracle, live, None, used, z, 0) == (0, 0)
    assert evict_both(oracle, live, np.ones(3000, np.int32), used, np.full(10, -1, np.int32), 0) == (0, 0)
    # equal stamps everywhere: exactly the ten lowest slots go
    n_free, n_ev = evict_both(oracle, live, None, used, np.full(10, -1, np.int32), 0)
    assert (n_free, n_ev) == (10, 10)


def test_steady_state_past_capacity(oracle):
    """Ten decoding steps over a pool that is full from the third step on.  Per step, on the device: norms ->
    layer-mean search -> decision -> remap (layer-shared table, reference counts) -> last-use stamps of the partners
    -> the references of the requests that end now are dropped -> eviction -> admission -> metadata of the admitted
    blocks.  The oracle runs the same step on its own copy of the state; every piece of state is compared after
    every step."""
    w = synth.scaled(synth.WORKLOADS[2], name="steady", L=2, P=96, Q=24, T=16, H=2, planted_frac=0.0, R=1, E=24, seed=41)
    say(f"{w.name}: P={w.P} Q={w.Q}, 10 steps, a block lives 3 steps")
    L, P, Q, NB = w.L, w.P, w.Q, w.P + w.Q
    gen = torch.Generator(device=DEV)
    gen.manual_seed(9)
    kv = lambda n: torch.randn((L, n, w.T, w.H, 128), generator=gen, device=DEV, dtype=torch.float32).to(torch.float16)
    kp, vp = kv(P), kv(P)
    live = torch.zeros(P, dtype=torch.uint8, device=DEV)
    live[:40] = 1                                              # 40 resident blocks to start with, referenced once each
    refc = torch.zeros(NB, dtype=torch.int32, device=DEV)
    refc[:40] = 1
    stamp = torch.zeros(P, dtype=torch.int32, device=DEV)
    pk, pv = rc.rc_block_norms(kp, vp, 0)
    qids = (P + torch.arange(Q, dtype=torch.int32, device=DEV)).contiguous()
    table = qids.reshape(1, 1, Q).clone()
    thr = parity.dist_tol(w.T, w.H, 128) * 30                  # noisy copies (sigma 0.02) are far below, fresh blocks far above
    # oracle-side state
    o = dict(kp=synth.bits(kp).copy(), vp=synth.bits(vp).copy(), live=live.cpu().numpy().copy(), refc=refc.cpu().numpy().copy(),
             stamp=stamp.cpu().numpy().copy())
    held = []                                                  # per step: the block every query's table entry ended up on
    full_steps = 0
    for step in range(1, 11):
        # new blocks: a third are noisy copies of blocks that are live right now, the rest fresh
        lv_now = np.flatnonzero(o["live"])
        kq, vq = kv(Q), kv(Q)
        ncopy = Q // 3
        src = torch.as_tensor(lv_now[np.random.RandomState(step).choice(lv_now.size, ncopy, replace=False)], device=DEV)
        kq[:, :ncopy] = (kp[:, src].float() + 0.02 * torch.randn(kp[:, src].shape, generator=gen, device=DEV)).to(torch.float16)
        vq[:, :ncopy] = (vp[:, src].float() + 0.02 * torch.randn(vp[:, src].shape, generator=gen, device=DEV)).to(torch.float16)
        qk, qv = rc.rc_block_norms(kq, vq, 0)
        m = rc.rc_match_blocks_layer_mean(kq, vq, qk, qv, kp, vp, pk, pv, live, thr)
        dec = m["match_idx"]
        refc[P:] = 1                                           # every new block starts with its owner's reference
        rm = rc.rc_remap_block_table(table, qids, None, dec.reshape(1, Q), P, NB, refc.reshape(1, NB), in_place=False)
        refc = rm["refcount"].reshape(NB).contiguous()
        rc.rc_pool_touch(dec, step, stamp)
        if len(held) >= 3:                                     # the requests of three steps ago end: their references go
            rc.rc_refcount_release(held[-3], refc)
        ev = rc.rc_pool_evict(live, refc[:P].contiguous(), stamp, dec)
        ad = rc.rc_pool_admit(kq, vq, qk, qv, kp, vp, pk, pv, live, dec)
        rc.rc_pool_touch(ad["slot_of_query"], step, stamp)
        pool_refc = refc[:P].contiguous()
        rc.rc_pool_touch(ad["slot_of_query"], 1, pool_refc)
        refc = torch.cat([pool_refc, torch.zeros(Q, dtype=torch.int32, device=DEV)])
        where = torch.where(dec >= 0, dec, ad["slot_of_query"]).contiguous()   # (-1: the block found no room and is lost)
        held.append(where)
        torch.cuda.synchronize()

        # ---- the same step on the oracle's state
        a = [synth.bits(x) for x in (kq, vq)]
        om = oracle.layer_mean(0, a[0], a[1], o["kp"], o["vp"], o["live"], thr, want_dist=True)
        gd = dec.cpu().numpy()
        gm = {k: v.cpu().numpy() for k, v in m.items()}
        parity.check_layer_mean(gm, om, thr, parity.dist_lookup(om["dist"], gm["best_idx"]), parity.dist_tol(w.T, w.H, 128))
        assert np.array_equal(gd, om["match_idx"])
        assert (gd[:ncopy] == src.cpu().numpy()).all() and (gd[ncopy:] == -1).all()
        o["refc"][P:] = 1
        orm = oracle.remap(table.cpu().numpy(), qids.cpu().numpy(), None, gd[None], P, NB, o["refc"][None])
        o["refc"] = orm["refcount"][0].copy()
        oracle.pool_touch(gd, step, o["stamp"])
        if len(held) > 3:
            oracle.refcount_release(held[-4].cpu().numpy(), o["refc"])
        pr_ = o["refc"][:P].copy()
        n_free, n_ev = oracle.pool_evict(o["live"], pr_, o["stamp"], gd)
        oqk, oqv = oracle.block_norms(0, 0, a[0], a[1])
        opk, opv = oracle.block_norms(0, 0, o["kp"], o["vp"])
        slot, n_adm = oracle.pool_admit(a[0], a[1], oqk, oqv, o["kp"], o["vp"], opk, opv, o["live"], gd)
        oracle.pool_touch(slot, step, o["stamp"])
        oracle.pool_touch(slot, 1, pr_)
        o["refc"] = np.concatenate([pr_, np.zeros(Q, np.int32)])
        # ---- compare the state, bit by bit
        assert (int(ev["n_free"].item()), int(ev["n_evicted"].item())) == (n_free, n_ev)
        assert np.array_equal(ad["slot_of_query"].cpu().numpy(), slot) and int(ad["n_admitted"].item()) == n_adm
        assert np.array_equal(live.cpu().numpy(), o["live"]) and np.array_equal(stamp.cpu().numpy(), o["stamp"])
        assert np.array_equal(refc.cpu().numpy(), o["refc"])
        assert np.array_equal(synth.bits(kp), o["kp"]) and np.array_equal(synth.bits(vp), o["vp"])
        n_live = int(o["live"].sum())
        full_steps += n_live == P
        say(f"step {step}: matched {int((gd >= 0).sum())}, evicted {n_ev}, admitted {n_adm}, live {n_live}/{P}")
        if step >= 5:
            assert n_ev > 0 and n_adm == Q - ncopy               # the steady state: what leaves makes room for what comes
    assert full_steps >= 3
