"""Parity of the HIP path (through the C ABI) with the CPU oracle.  Needs a real MI355X."""
import sys

import numpy as np
import pytest
import torch

from paper_2507_21433_amd import binding as rc
from paper_2507_21433_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
NORM_RTOL = 2e-5   # fp32 sum of exact products: (chain 64 + tree 9) * 2^-24 ~ 4.4e-6 worst case


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def dcode(w):
    return 0 if w.dtype == "f16" else 1


def run_gpu_match(pr, w, live=None, want_second=True):
    qk, qv = rc.rc_block_norms(pr["kq"], pr["vq"], w.mode)
    pk, pv = rc.rc_block_norms(pr["kp"], pr["vp"], w.mode)
    out = rc.rc_match_blocks(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, live, w.tau, w.mode,
                             want_second=want_second)
    torch.cuda.synchronize()
    return {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}, (qk, qv, pk, pv)


def oracle_match(oracle, pr, w, live, layers=None, queries=None, want_scores=True):
    sl = slice(None) if layers is None else layers
    qs = slice(None) if queries is None else queries
    a = [synth.bits(pr[n][sl][:, qs] if n[1] == "q" else pr[n][sl]) for n in ("kq", "vq", "kp", "vp")]
    lv = None if live is None else live[sl].cpu().numpy()
    return oracle.match(dcode(w), w.mode, *a, lv, w.tau, want_scores=want_scores)


def full_check(oracle, w, pr, live_t):
    gpu, _ = run_gpu_match(pr, w, live_t)
    orc = oracle_match(oracle, pr, w, live_t)
    rep = parity.check_match(gpu, orc, w.tau, parity.score_lookup(orc["scores"], gpu["best_idx"]))
    say(f"{w.name}: {rep}")
    return gpu, orc, rep


# ------------------------------------------------------------------ norms
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("T,H,mode", [(16, 8, 0), (32, 8, 0), (16, 8, 1), (32, 8, 1), (16, 3, 1), (16, 16, 1), (32, 5, 0)])
def test_norms(oracle, dtype, T, H, mode):
    say(f"norms dtype={dtype} T={T} H={H} mode={mode}")
    g = torch.Generator(device="cpu").manual_seed(7)
    L, n = 3, 37
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    # layers sit in a larger allocation (layer_stride > n*D); scale differs per block
    scale = (0.25 + 4 * torch.rand(L, n + 2, 1, 1, 1, generator=g))
    k = (torch.randn(L, n + 2, T, H, 128, generator=g) * scale).to(tdt).to(DEV)
    v = (torch.randn(L, n + 2, T, H, 128, generator=g) * scale).to(tdt).to(DEV)
    k[1, 5] = 0
    kk, vv = k[:, :n], v[:, :n]
    ksq, vsq = rc.rc_block_norms(kk, vv, mode)
    torch.cuda.synchronize()
    ok, ov = oracle.block_norms(0 if dtype == "f16" else 1, mode, synth.bits(kk), synth.bits(vv))
    assert np.allclose(ksq.cpu().numpy(), ok, rtol=NORM_RTOL, atol=0)
    assert np.allclose(vsq.cpu().numpy(), ov, rtol=NORM_RTOL, atol=0)
    assert (ksq[1, 5] == 0).all()


# ------------------------------------------------------------------ match
def test_cfg1_tiny(oracle):
    w = synth.WORKLOADS[1]
    say(w.name)
    pr = synth.make_problem(w, DEV)
    gpu, orc, rep = full_check(oracle, w, pr, pr["live"])
    plan = pr["plan"]
    want = np.full(w.Q, -1)
    want[plan.planted_slots] = plan.planted_targets
    assert np.array_equal(gpu["match_idx"][0], want)
    assert rep["matched"] == 8


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("P,Q", [(700, 300), (256, 256), (257, 1), (1, 5), (513, 257),
                                 (300, 64), (300, 65), (259, 128), (300, 129)])   # the last four: the edges of the 64- and 128-column tiles
def test_match_ragged_tiles(oracle, dtype, P, Q):
    # several pool tiles and query tiles with ragged tails, dead blocks, bit-identical pool blocks
    w = synth.scaled(synth.WORKLOADS[2], name=f"ragged_{dtype}_{P}x{Q}", L=2, P=P, Q=Q, dtype=dtype,
                     planted_frac=0.3 if P >= Q else 0.0, R=1, E=P + Q, seed=11)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    live = pr["live"].clone()
    if P > 8:
        live[0, 3] = 0
        live[1, P - 1] = 0
        tgt = int(pr["plan"].planted_targets[0]) if pr["plan"].planted_targets.size else 0
        live[0, tgt] = 0                      # a planted partner is dead in layer 0
        pr["kp"][:, P - 2] = pr["kp"][:, 1]   # bit-identical pool blocks far apart: lowest index must win
        pr["vp"][:, P - 2] = pr["vp"][:, 1]
        pr["kq"][:, 0] = pr["kp"][:, 1]
        pr["vq"][:, 0] = pr["vp"][:, 1]
    gpu, orc, rep = full_check(oracle, w, pr, live)
    if P > 8:
        assert gpu["best_idx"][1, 0] == 1 and gpu["match_idx"][1, 0] == 1
        assert abs(gpu["best_score"][1, 0] - 1.0) < 1e-5 and abs(gpu["second_score"][1, 0] - 1.0) < 1e-5


@pytest.mark.parametrize("L,P,Q", [(48, 513, 257), (80, 700, 64), (70, 513, 128)])
def test_match_many_layers_whole_tiles(oracle, L, P, Q):
    # more than 128 tiles: every tile is computed by one workgroup (no split of the reduction), with the
    # 256-, 64- and 128-column tile; the small cases above all take the split path
    w = synth.scaled(synth.WORKLOADS[2], name=f"whole_tiles_L{L}_{P}x{Q}", L=L, P=P, Q=Q, planted_frac=0.3, R=1,
                     E=P + Q, seed=13)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    live = pr["live"].clone()
    live[:, 5] = 0
    live[0, int(pr["plan"].planted_targets[0])] = 0
    pr["kp"][:, P - 2] = pr["kp"][:, 1]       # bit-identical pool blocks in different tiles: lowest index must win
    pr["vp"][:, P - 2] = pr["vp"][:, 1]
    pr["kq"][:, 0] = pr["kp"][:, 1]
    pr["vq"][:, 0] = pr["vp"][:, 1]
    gpu, orc, rep = full_check(oracle, w, pr, live)
    assert (gpu["best_idx"][:, 0] == 1).all() and (gpu["match_idx"][:, 0] == 1).all()


@pytest.mark.parametrize("mode,H", [(0, 1), (1, 2)])
def test_match_many_rounds_tiles_change_hands(oracle, mode, H):
    # 16 rounds of tiles and more: the last tenth of every XCD's list of tiles can be taken over by the workgroups of
    # the XCDs that are through with theirs.  Every tile must still be computed exactly once: the call equals, bit
    # for bit, the same layers scored 20 at a time (two rounds, the fixed schedule), and sampled queries equal the
    # oracle's search.
    L, P, Q = 260, 513, 1300
    w = synth.scaled(synth.WORKLOADS[2 if mode == 0 else 5], name=f"many_rounds_mode{mode}_L{L}_{P}x{Q}", L=L, P=P, Q=Q,
                     T=16, H=H, planted_frac=0.3, R=1, E=P + Q, seed=21)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    live = pr["live"].clone()
    live[:, 9] = 0
    for rep in range(3):  # who takes which tile differs from run to run
        whole, _ = run_gpu_match(pr, w, live)
        for l0 in range(0, L, 20):
            part = {n: pr[n][l0:l0 + 20] for n in ("kq", "vq", "kp", "vp")}
            some, _ = run_gpu_match(part, synth.scaled(w, L=20), live[l0:l0 + 20])
            for k in ("best_idx", "match_idx"):
                assert np.array_equal(whole[k][l0:l0 + 20], some[k]), (rep, l0, k)
            for k in ("best_score", "second_score"):
                assert np.array_equal(whole[k][l0:l0 + 20].view(np.uint32), some[k].view(np.uint32)), (rep, l0, k)
    layers = [0, 131, 259]
    queries = np.arange(0, Q, 31)
    orc = oracle_match(oracle, pr, w, live, layers=layers, queries=queries)
    sub = {k: whole[k][layers][:, queries] for k in whole}
    rep = parity.check_match(sub, orc, w.tau, parity.score_lookup(orc["scores"], sub["best_idx"]))
    say(f"{w.name}: {rep}")


def test_match_split_shapes(oracle):
    # the split of the reduction at its extremes: one tile over 64 shares (8 steps each), 128 tiles over 2
    # shares (a whole tensor each), head counts whose step count is not a power of two
    for (L, P, Q, T, H) in [(1, 200, 30, 16, 8), (32, 1000, 40, 16, 8), (1, 300, 257, 16, 3), (2, 257, 5, 32, 5),
                            (1, 100, 7, 16, 1)]:
        w = synth.scaled(synth.WORKLOADS[2], name=f"split_L{L}_{P}x{Q}_T{T}_H{H}", L=L, P=P, Q=Q, T=T, H=H,
                         planted_frac=0.3, R=1, E=P + Q, seed=19)
        say(w.name)
        pr = synth.make_problem(w, DEV)
        live = pr["live"].clone()
        live[:, 3] = 0
        full_check(oracle, w, pr, live)


def test_match_degenerate_blocks(oracle):
    # zero query, zero pool block, zero V only, huge and tiny norms, tau = 1 on exact duplicates
    w = synth.scaled(synth.WORKLOADS[2], name="degenerate", L=1, P=300, Q=40, planted_frac=0.0, R=1, E=340, seed=5,
                     tau=0.99999)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    pr["kq"][0, 0] = 0
    pr["vq"][0, 0] = 0                     # all-zero query: score 0, no NaN, no match
    pr["kp"][0, 7] = 0
    pr["vp"][0, 7] = 0                     # all-zero pool block
    pr["vq"][0, 1] = 0                     # V zero, K alive
    pr["kq"][0, 2] = pr["kp"][0, 11]
    pr["vq"][0, 2] = pr["vp"][0, 11]       # exact duplicate
    pr["kp"][0, 20] = (pr["kp"][0, 20].float() * 30).half()     # K norm 30x the V norm
    pr["kq"][0, 3] = pr["kp"][0, 20]
    pr["vq"][0, 3] = pr["vp"][0, 20]
    pr["vp"][0, 21] = (pr["vp"][0, 21].float() / 64).half()     # V norm tiny
    pr["kq"][0, 4] = pr["kp"][0, 21]
    pr["vq"][0, 4] = pr["vp"][0, 21]
    gpu, orc, rep = full_check(oracle, w, pr, None)
    assert np.isfinite(gpu["best_score"]).all()
    assert gpu["match_idx"][0, 0] == -1 and abs(gpu["best_score"][0, 0]) < 1e-6
    assert gpu["best_idx"][0, 2] == 11 and gpu["best_idx"][0, 3] == 20 and gpu["best_idx"][0, 4] == 21


def test_match_no_live_and_empty(oracle):
    w = synth.scaled(synth.WORKLOADS[2], name="nolive", L=2, P=64, Q=9, planted_frac=0.0, R=1, E=73, seed=6)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    live = torch.zeros_like(pr["live"])
    live[1, 10] = 1
    gpu, orc, rep = full_check(oracle, w, pr, live)
    assert (gpu["best_idx"][0] == -1).all() and (gpu["best_idx"][1] == 10).all()
    assert np.isneginf(gpu["second_score"]).all()
    # P == 0: nothing to pick from
    qk, qv = rc.rc_block_norms(pr["kq"], pr["vq"], 0)
    empty = pr["kp"][:, :0]
    out = rc.rc_match_blocks(pr["kq"], pr["vq"], qk, qv, empty, empty, qk[:, :0].contiguous(), qk[:, :0].contiguous(),
                             None, 0.5, 0)
    torch.cuda.synchronize()
    assert (out["best_idx"] == -1).all() and (out["match_idx"] == -1).all() and torch.isneginf(out["best_score"]).all()
    # Q == 0: nothing is launched, nothing is written
    out = rc.rc_match_blocks(pr["kq"][:, :0], pr["vq"][:, :0], qk[:, :0].contiguous(), qk[:, :0].contiguous(),
                             pr["kp"], pr["vp"], qk, qv, None, 0.5, 0)
    assert out["best_idx"].numel() == 0


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_per_head_mode(oracle, dtype):
    w = synth.scaled(synth.WORKLOADS[5], name=f"perhead_{dtype}", L=2, P=300, Q=70, dtype=dtype, R=2, E=185, seed=13)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    # adversarial pair: seven heads exact, one head noisy -> the block score would match, per-head-all must not
    g = torch.Generator(device=DEV).manual_seed(3)
    pr["kq"][0, 1] = pr["kp"][0, 17]
    pr["vq"][0, 1] = pr["vp"][0, 17]
    for q, src in (("kq", "kp"), ("vq", "vp")):
        noisy = pr[src][0, 17, :, 3].float() + 0.5 * torch.randn(w.T, w.Dh, device=DEV, generator=g)
        pr[q][0, 1, :, 3] = noisy.to(w.torch_dtype)
    gpu, orc, rep = full_check(oracle, w, pr, pr["live"])
    assert gpu["best_idx"][0, 1] == 17 and gpu["match_idx"][0, 1] == -1
    wb = synth.scaled(w, mode=0)
    gb, _ = run_gpu_match(pr, wb, pr["live"])
    assert gb["match_idx"][0, 1] == 17
    plan = pr["plan"]
    slots = plan.planted_slots[plan.planted_slots != 1]
    assert (gpu["match_idx"][1][slots] >= 0).all()


def test_per_head_many_layers_whole_tiles(oracle):
    # more than one round of tiles: one workgroup per tile walks all heads and keeps the running minimum in
    # 16-bit fixed point (the small per-head cases take the one-share-per-head path instead)
    w = synth.scaled(synth.WORKLOADS[5], name="perhead_whole_tiles", L=90, P=513, Q=40, T=16, R=2, E=300, seed=15)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    live = pr["live"].clone()
    live[:, 7] = 0
    full_check(oracle, w, pr, live)


def test_per_head_scores_do_not_depend_on_the_path():
    # the same layer scored inside a call of 90 layers (whole tiles, running minimum in 16-bit fixed point) and in a
    # call of its own (one share per head, minimum taken by the selection kernel): identical bits, identical picks
    w = synth.scaled(synth.WORKLOADS[5], name="perhead_paths", L=90, P=513, Q=40, T=16, R=2, E=300, seed=16)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    many, _ = run_gpu_match(pr, w, pr["live"])
    for l in (0, 37, 89):
        one = {n: pr[n][l:l + 1] for n in ("kq", "vq", "kp", "vp")}
        alone, _ = run_gpu_match(one, synth.scaled(w, L=1), pr["live"][l:l + 1])
        for k in ("best_score", "second_score"):
            assert np.array_equal(many[k][l].view(np.uint32), alone[k][0].view(np.uint32)), (l, k)
        for k in ("best_idx", "match_idx"):
            assert np.array_equal(many[k][l], alone[k][0]), (l, k)
        # multiples of 1/32767
        assert np.array_equal(np.round(many["best_score"][l].astype(np.float64) * 32767) / 32767,
                              many["best_score"][l].astype(np.float64).round(12)) or \
            np.abs(np.round(many["best_score"][l].astype(np.float64) * 32767) / 32767 - many["best_score"][l]).max() < 1e-7


def test_per_head_T16_H4(oracle):
    w = synth.scaled(synth.WORKLOADS[5], name="perhead_T16_H4", L=1, P=130, Q=33, T=16, H=4, R=1, E=163, seed=14)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    full_check(oracle, w, pr, pr["live"])


def test_clustered_near_ties(oracle):
    # runner-up within 2e-3 of the best is common here: exercises the ambiguous-query rule
    w = synth.scaled(synth.WORKLOADS[3], name="clustered_small", L=1, P=1024, Q=96, n_centroids=8, R=4, E=280)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    gpu, orc, rep = full_check(oracle, w, pr, pr["live"])
    assert rep["near_tie"] > 0


def test_layer_stride_padding(oracle):
    # layers of a tensor separated by unrelated data
    w = synth.scaled(synth.WORKLOADS[2], name="strided", L=3, P=260, Q=20, R=1, E=280, seed=21)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    big = {n: torch.randn((w.L, pr[n].shape[1] + 3, w.T, w.H, w.Dh), device=DEV).to(w.torch_dtype) for n in ("kq", "vq", "kp", "vp")}
    view = {}
    for n in big:
        big[n][:, :pr[n].shape[1]] = pr[n]
        view[n] = big[n][:, :pr[n].shape[1]]
    pr2 = dict(pr, **view)
    gpu, _ = run_gpu_match(pr2, w, pr["live"])
    ref, _ = run_gpu_match(pr, w, pr["live"])
    for k in ref:
        assert np.array_equal(gpu[k], ref[k]), k
    orc = oracle_match(oracle, pr, w, pr["live"])
    parity.check_match(gpu, orc, w.tau, parity.score_lookup(orc["scores"], gpu["best_idx"]))


def test_deterministic(oracle):
    w = synth.scaled(synth.WORKLOADS[3], name="determinism", L=2, P=600, Q=300, n_centroids=8, R=4, E=280)
    say(w.name)
    pr = synth.make_problem(w, DEV)
    a, _ = run_gpu_match(pr, w, pr["live"])
    for _ in range(3):
        b, _ = run_gpu_match(pr, w, pr["live"])
        for k in a:
            assert np.array_equal(a[k], b[k]), k


# ------------------------------------------------------------------ remap
def gpu_remap(tables, qids, pids, match, P, NB, rc_in, in_place=False):
    t = lambda a, dt=torch.int32: None if a is None else torch.as_tensor(np.ascontiguousarray(a), dtype=dt, device=DEV)
    out = rc.rc_remap_block_table(t(tables), t(qids), t(pids), t(match), P, NB, t(rc_in), in_place=in_place)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


def assert_remap_equal(g, o):
    for k in ("tables", "refcount", "freed", "n_remapped"):
        assert np.array_equal(g[k], o[k]), k


@pytest.mark.parametrize("in_place", [False, True])
def test_remap_random(oracle, in_place):
    rng = np.random.RandomState(17)
    # small and large id ranges (decided in LDS / through global memory), tables of one and of several workgroups
    # per layer (counts finalized by the gathering workgroup / by a launch of its own), many small layers
    for case in range(10):
        L, P, Q, R, E = [(3, 40, 12, 5, 30), (2, 3000, 700, 9, 1031), (1, 50, 1, 1, 7), (4, 10, 64, 3, 4099),
                         (1, 5000, 2000, 64, 300), (2, 17, 9, 2, 1), (2, 20000, 8192, 8, 5003),
                         (1, 70000, 4500, 16, 4100), (1, 3000, 700, 40, 2000), (130, 50, 20, 2, 33)][case]
        say(f"remap random case {case} L={L} P={P} Q={Q} R={R} E={E} in_place={in_place}")
        NB = P + Q + 5
        ids = rng.permutation(NB)
        pids, qids = ids[:P].astype(np.int32), ids[P:P + Q].astype(np.int32)
        tables = rng.choice(np.concatenate([ids[:P + Q], [-1, NB + 3]]), size=(L, R, E)).astype(np.int32)
        refcount = np.stack([np.bincount(t[(t >= 0) & (t < NB)], minlength=NB) for t in tables]).astype(np.int32)
        refcount[:, qids[0]] += 1                       # a reference held outside the tables
        match = rng.randint(-1, P, size=(L, Q)).astype(np.int32)
        match[rng.rand(L, Q) < 0.4] = -1
        if Q > 3:
            match[:, 1] = match[:, 0]
            match[:, 3] = match[:, 0]                  # three queries share one target
            match[:, 2] = P + 7                        # out of range: treated as unmatched
        o = oracle.remap(tables, qids, pids, match, P, NB, refcount)
        g = gpu_remap(tables, qids, pids, match, P, NB, refcount, in_place)
        assert_remap_equal(g, o)


def test_remap_all_to_one_target(oracle):
    say("remap all queries to one target")
    P, Q, NB = 8, 1500, 1508
    tables = np.concatenate([np.arange(NB), np.arange(P, NB)]).astype(np.int32).reshape(1, 1, -1)
    refcount = np.bincount(tables.ravel(), minlength=NB).astype(np.int32)[None]
    match = np.full((1, Q), 5, dtype=np.int32)
    qids = (P + np.arange(Q)).astype(np.int32)
    o = oracle.remap(tables, qids, None, match, P, NB, refcount)
    g = gpu_remap(tables, qids, None, match, P, NB, refcount)
    assert_remap_equal(g, o)
    assert g["refcount"][0, 5] == 1 + 2 * Q and g["freed"].all()


def test_remap_every_entry_is_rewritten(oracle):
    # whole batches in which every entry names a matched query block: the list of a batch's hits is full
    say("remap: 40000 entries, all of them references to matched query blocks")
    rng = np.random.RandomState(23)
    P, Q, NB = 8, 4096, 8 + 4096
    qids = (P + rng.permutation(Q)).astype(np.int32)
    tables = qids[rng.randint(0, Q, size=(2, 1, 40000))].astype(np.int32)
    refcount = np.stack([np.bincount(t.ravel(), minlength=NB) for t in tables]).astype(np.int32)
    match = rng.randint(0, P, size=(2, Q)).astype(np.int32)
    o = oracle.remap(tables, qids, None, match, P, NB, refcount)
    g = gpu_remap(tables, qids, None, match, P, NB, refcount)
    assert_remap_equal(g, o)
    assert int(g["n_remapped"].sum()) == 80000 and g["freed"].all()


def test_remap_cfg4_tables_all_layers(oracle):
    # the high-concurrency table shape, all 64 layers: 64 tables x 776 entries, dead blocks, refcounts
    w = synth.WORKLOADS[4]
    say("remap cfg4 tables, 64 layers")
    plan = synth.make_plan(w)
    rng = np.random.RandomState(1)
    match = np.full((w.L, w.Q), -1, dtype=np.int32)
    match[:, plan.planted_slots] = plan.planted_targets
    match[:, plan.planted_slots[plan.live[plan.planted_targets] == 0]] = -1    # plants aimed at dead blocks stay
    flip = rng.rand(w.L, w.Q) < 0.05
    match[flip] = -1                                                          # layers differ a little
    tables = np.repeat(plan.tables[None], w.L, axis=0)
    refcount = np.repeat(plan.refcount[None], w.L, axis=0)
    o = oracle.remap(tables, plan.query_ids, None, match, w.P, w.NB, refcount)
    g = gpu_remap(tables, plan.query_ids, None, match, w.P, w.NB, refcount)
    assert_remap_equal(g, o)
    # invariant: tables only point at blocks that are still referenced, and never at dead ones
    for l in (0, 31, 63):
        t = g["tables"][l]
        assert (g["refcount"][l][t] >= 1).all()
        pool_refs = t[t < w.P]
        assert (plan.live[pool_refs] == 1).all()


def test_end_to_end_cfg1_remap(oracle):
    # norms -> match -> remap chained on the device, checked against the oracle chain
    w = synth.WORKLOADS[1]
    say("end to end cfg1")
    pr = synth.make_problem(w, DEV)
    qk, qv = rc.rc_block_norms(pr["kq"], pr["vq"], w.mode)
    pk, pv = rc.rc_block_norms(pr["kp"], pr["vp"], w.mode)
    m = rc.rc_match_blocks(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, pr["live"], w.tau, w.mode)
    out = rc.rc_remap_block_table(pr["tables"], pr["query_ids"], None, m["match_idx"], w.P, w.NB, pr["refcount"])
    torch.cuda.synchronize()
    orc = oracle_match(oracle, pr, w, pr["live"], want_scores=False)
    assert np.array_equal(m["match_idx"].cpu().numpy(), orc["match_idx"])
    o = oracle.remap(pr["tables"].cpu().numpy(), pr["query_ids"].cpu().numpy(), None, orc["match_idx"], w.P, w.NB,
                     pr["refcount"].cpu().numpy())
    assert_remap_equal({k: v.cpu().numpy() for k, v in out.items()}, o)
    assert int(out["n_remapped"].sum()) == 8 and int(out["freed"].sum()) == 8


# ------------------------------------------------------------------ argument errors (no launch happens)
def test_argument_errors():
    say("argument errors")
    w = synth.scaled(synth.WORKLOADS[1], P=8, Q=4, E=8)
    pr = synth.make_problem(w, DEV)
    qk, qv = rc.rc_block_norms(pr["kq"], pr["vq"], 0)
    pk, pv = rc.rc_block_norms(pr["kp"], pr["vp"], 0)
    with pytest.raises(rc.RcError) as e:
        rc.rc_match_blocks(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, None, 0.5, 0,
                           workspace=torch.empty(16, dtype=torch.uint8, device=DEV))
    assert e.value.code == 3
    with pytest.raises(rc.RcError) as e:
        rc.rc_match_blocks(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, None, float("nan"), 0)
    assert e.value.code == 1
    with pytest.raises(rc.RcError) as e:
        rc.rc_block_norms(pr["kq"], pr["vq"], 7)
    assert e.value.code == 2
    bad = torch.zeros((1, 2, 16, 8, 64), dtype=torch.float16, device=DEV)
    with pytest.raises(rc.RcError) as e:
        rc.rc_block_norms(bad, bad, 0)
    assert e.value.code == 2
