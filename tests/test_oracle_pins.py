"""Pins of the CPU oracle against things that are not the oracle.

Each test fixes the oracle to a fact the paper or plain mathematics determines:
library bit decoders, integer closed forms, the squared-distance expansion of
Sec. IV-A Stage 2, hand-worked pairs and tables (tests/golden), statistical laws
of the synthetic workloads, and brute force written with a different formula.
No GPU is involved.
"""
import json
import os

import numpy as np
import pytest
import torch

from paper_2507_21433_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def enc(x, dtype):
    """float array -> uint16 bit patterns through a library encoder (numpy fp16 / torch bf16)."""
    x = np.asarray(x, dtype=np.float32)
    if dtype == 0:
        return x.astype(np.float16).view(np.uint16)
    return torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def dec(bits, dtype):
    """uint16 bit patterns -> float64 through a library decoder."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == 0:
        return bits.view(np.float16).astype(np.float64)
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()


def blk(x, T, H, Dh, dtype):
    """1 layer, n blocks: [n][D] floats -> [1][n][T][H][Dh] bits."""
    x = np.asarray(x, dtype=np.float32)
    return enc(x, dtype).reshape(1, -1, T, H, Dh)


# ---------------------------------------------------------------- decoding
@pytest.mark.parametrize("dtype", [0, 1])
def test_decode_all_bit_patterns(oracle, dtype):
    bits = np.arange(65536, dtype=np.uint16)
    mine = oracle.decode(dtype, bits)
    ref = dec(bits, dtype)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(mine), nan)
    assert np.array_equal(mine[~nan], ref[~nan])
    assert np.array_equal(np.signbit(mine[~nan]), np.signbit(ref[~nan]))


# ---------------------------------------------------------------- norms
@pytest.mark.parametrize("dtype", [0, 1])
def test_norm_integer_closed_form(oracle, dtype):
    # 1..16 -> sum of squares n(n+1)(2n+1)/6 = 1496; ones -> D; a single 3 -> 9.
    T, H, Dh = 2, 2, 4
    D = T * H * Dh
    x = np.stack([np.arange(1, D + 1), np.ones(D), np.eye(D)[5] * 3.0, np.zeros(D)])
    k = blk(x, T, H, Dh, dtype)
    v = blk(2 * x, T, H, Dh, dtype)
    ksq, vsq = oracle.block_norms(dtype, oracle.BLOCK, k, v)
    assert ksq.tolist() == [[1496.0, 16.0, 9.0, 0.0]]
    assert vsq.tolist() == [[4 * 1496.0, 64.0, 36.0, 0.0]]


def test_norm_per_head_slices_and_layers(oracle):
    # Head h of a [T][H][Dh] block is x[:, h, :]; checked with numpy's own reshape on two layers.
    rng = np.random.RandomState(5)
    L, n, T, H, Dh = 2, 3, 4, 3, 8
    x = rng.randint(-8, 9, size=(L, n, T, H, Dh)).astype(np.float32)
    y = rng.randint(-8, 9, size=(L, n, T, H, Dh)).astype(np.float32)
    ksq, vsq = oracle.block_norms(0, oracle.PER_HEAD_ALL, enc(x, 0), enc(y, 0))
    assert ksq.shape == (L, n, H)
    assert np.array_equal(ksq, (x.astype(np.float64) ** 2).sum(axis=(2, 4)))
    assert np.array_equal(vsq, (y.astype(np.float64) ** 2).sum(axis=(2, 4)))
    kb, vb = oracle.block_norms(0, oracle.BLOCK, enc(x, 0), enc(y, 0))
    assert np.array_equal(kb, ksq.sum(axis=2)) and np.array_equal(vb, vsq.sum(axis=2))


# ---------------------------------------------------------------- pair scores
@pytest.mark.parametrize("dtype", [0, 1])
def test_golden_pairs(oracle, dtype):
    cases = json.load(open(os.path.join(GOLD, "pair_scores_handworked.json")))["cases"]
    for c in cases:
        T, H, Dh = c["T"], c["H"], c["Dh"]
        a = [blk([c[n]], T, H, Dh, dtype) for n in ("kq", "vq", "kp", "vp")]
        z = np.zeros(1, dtype=np.int32)
        s_block = oracle.score_pairs(dtype, oracle.BLOCK, *a, z, z, z)[0]
        s_head = oracle.score_pairs(dtype, oracle.PER_HEAD_ALL, *a, z, z, z)[0]
        assert s_block == pytest.approx(c["block"], abs=1e-14), c["name"]
        assert s_head == pytest.approx(c["per_head"], abs=1e-14), c["name"]
        # the search must report the same numbers as the from-scratch pair routine
        for mode, want in ((oracle.BLOCK, c["block"]), (oracle.PER_HEAD_ALL, c["per_head"])):
            r = oracle.match(dtype, mode, a[0], a[1], a[2], a[3], None, -10.0, want_scores=True)
            assert r["scores"][0, 0, 0] == pytest.approx(want, abs=1e-14)
            assert r["best_score"][0, 0] == pytest.approx(want, abs=1e-14)


@pytest.mark.parametrize("dtype", [0, 1])
def test_expansion_identity_vs_direct_distance(oracle, dtype):
    # |x-y|^2 computed by subtracting and squaring must equal |x|^2 + |y|^2 - 2 x.y  (Stage 2 expansion),
    # with x.y recovered from the oracle's cosine.  V is a copy (cos 1) so s = (cosK + 1)/2.
    rng = np.random.RandomState(11)
    T, H, Dh = 2, 2, 4
    D = T * H * Dh
    for _ in range(20):
        x = enc(rng.randn(D), dtype)
        y = enc(rng.randn(D), dtype)
        kq, kp = x.reshape(1, 1, T, H, Dh), y.reshape(1, 1, T, H, Dh)
        ones = blk([np.ones(D)], T, H, Dh, dtype)
        z = np.zeros(1, dtype=np.int32)
        s = oracle.score_pairs(dtype, oracle.BLOCK, kq, ones, kp, ones, z, z, z)[0]
        nx, _ = oracle.block_norms(dtype, oracle.BLOCK, kq, ones)
        ny, _ = oracle.block_norms(dtype, oracle.BLOCK, kp, ones)
        nx, ny = nx[0, 0], ny[0, 0]
        xy = (2 * s - 1) * np.sqrt(nx * ny)
        direct = oracle.sqdist(dtype, x, y)
        assert direct == pytest.approx(nx + ny - 2 * xy, rel=1e-12, abs=1e-12)
        # and against numpy on library-decoded values
        xd, yd = dec(x, dtype), dec(y, dtype)
        assert direct == pytest.approx(((xd - yd) ** 2).sum(), rel=1e-13)
        assert xy == pytest.approx(float(xd @ yd), rel=1e-11, abs=1e-11)
        # unit vectors: |x^ - y^|^2 = 2 - 2 cos
        cos = 2 * s - 1
        assert ((xd / np.sqrt(nx) - yd / np.sqrt(ny)) ** 2).sum() == pytest.approx(2 - 2 * cos, abs=1e-12)


@pytest.mark.parametrize("mode", [0, 1])
def test_duplicate_is_exactly_one_and_orthogonal_exactly_zero(oracle, mode):
    rng = np.random.RandomState(3)
    T, H, Dh = 16, 8, 128
    D = T * H * Dh
    x = rng.randn(2, D).astype(np.float32)
    k, v = blk(x[:1], T, H, Dh, 0), blk(x[1:], T, H, Dh, 0)
    z = np.zeros(1, dtype=np.int32)
    assert oracle.score_pairs(0, mode, k, v, k.copy(), v.copy(), z, z, z)[0] == 1.0
    # disjoint supports: even dims vs odd dims
    a, b = x.copy(), x.copy()
    a[:, 0::2] = 0
    b[:, 1::2] = 0
    s = oracle.score_pairs(0, mode, blk(a[:1], T, H, Dh, 0), blk(a[1:], T, H, Dh, 0),
                           blk(b[:1], T, H, Dh, 0), blk(b[1:], T, H, Dh, 0), z, z, z)[0]
    assert s == 0.0
    # all-zero query: defined as 0, never NaN, never a match for tau > 0
    zero = np.zeros((1, 1, T, H, Dh), dtype=np.uint16)
    r = oracle.match(0, mode, zero, zero, k, v, None, 0.5)
    assert r["best_score"][0, 0] == 0.0 and r["match_idx"][0, 0] == -1


def test_noisy_copy_law_and_fresh_pairs(oracle):
    # x ~ N(0,1)^D, y = x + N(0, sigma^2): cos -> 1/sqrt(1 + sigma^2); independent pairs: cos ~ N(0, 1/D).
    rng = np.random.RandomState(9)
    T, H, Dh = 16, 8, 128
    D = T * H * Dh
    pool = rng.randn(4, 2, D).astype(np.float32)
    for sigma in (0.1, 0.15):
        q = pool + sigma * rng.randn(4, 2, D).astype(np.float32)
        for i in range(4):
            z = np.zeros(1, dtype=np.int32)
            s = oracle.score_pairs(0, 0, blk(q[i, :1], T, H, Dh, 0), blk(q[i, 1:], T, H, Dh, 0),
                                   blk(pool[i, :1], T, H, Dh, 0), blk(pool[i, 1:], T, H, Dh, 0), z, z, z)[0]
            assert s == pytest.approx(1 / np.sqrt(1 + sigma ** 2), abs=3e-3)
    z = np.zeros(1, dtype=np.int32)
    s = oracle.score_pairs(0, 0, blk(pool[0, :1], T, H, Dh, 0), blk(pool[0, 1:], T, H, Dh, 0),
                           blk(pool[1, :1], T, H, Dh, 0), blk(pool[1, 1:], T, H, Dh, 0), z, z, z)[0]
    assert abs(s) < 6 / np.sqrt(D)


def test_per_head_rule_adversarial(oracle):
    # Seven heads exact copies, one head with sigma = 0.5 noise: the whole-block cosine stays
    # near 8/sqrt(8 * 8.25) = 0.985 (would match at 0.95), the noisy head alone is near
    # 1/sqrt(1.25) = 0.894, so "all heads must clear tau" must refuse the pair.
    rng = np.random.RandomState(21)
    T, H, Dh = 16, 8, 128
    p = rng.randn(2, T, H, Dh).astype(np.float32)
    q = p.copy()
    q[:, :, 3, :] += 0.5 * rng.randn(2, T, Dh).astype(np.float32)
    a = [blk(t.reshape(1, -1), T, H, Dh, 0) for t in (q[0], q[1], p[0], p[1])]
    rb = oracle.match(0, 0, *a, None, 0.95)
    rh = oracle.match(0, 1, *a, None, 0.95)
    assert rb["best_score"][0, 0] == pytest.approx(8 / np.sqrt(8 * 8.25), abs=4e-3) and rb["match_idx"][0, 0] == 0
    assert rh["best_score"][0, 0] == pytest.approx(1 / np.sqrt(1.25), abs=1e-2) and rh["match_idx"][0, 0] == -1


# ---------------------------------------------------------------- search
def brute_scores(kq, vq, kp, vp, dtype, mode):
    """Score matrix by a different route: cos = 1 - |x^ - y^|^2 / 2 on library-decoded values."""
    L, Q, T, H, Dh = kq.shape
    P = kp.shape[1]
    d = [dec(a, dtype).reshape(a.shape) for a in (kq, vq, kp, vp)]
    out = np.zeros((L, Q, P))

    def cos(x, y):
        nx, ny = np.sqrt((x * x).sum()), np.sqrt((y * y).sum())
        if nx == 0 or ny == 0:
            return 0.0
        return 1.0 - (((x / nx) - (y / ny)) ** 2).sum() / 2.0

    for l in range(L):
        for q in range(Q):
            for p in range(P):
                if mode == 0:
                    out[l, q, p] = 0.5 * (cos(d[0][l, q], d[2][l, p]) + cos(d[1][l, q], d[3][l, p]))
                else:
                    out[l, q, p] = min(0.5 * (cos(d[0][l, q, :, h], d[2][l, p, :, h]) +
                                              cos(d[1][l, q, :, h], d[3][l, p, :, h])) for h in range(H))
    return out


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("mode", [0, 1])
def test_match_vs_brute_force(oracle, dtype, mode):
    rng = np.random.RandomState(100 + 10 * dtype + mode)
    L, Q, P, T, H, Dh = 2, 5, 9, 2, 3, 4
    D = T * H * Dh
    kp, vp = rng.randn(L, P, D), rng.randn(L, P, D)
    kq, vq = rng.randn(L, Q, D), rng.randn(L, Q, D)
    kq[:, 0], vq[:, 0] = kp[:, 4] + 0.05 * rng.randn(L, D), vp[:, 4] + 0.05 * rng.randn(L, D)
    kq[:, 1], vq[:, 1] = kp[:, 7], vp[:, 7]
    a = [enc(t, dtype).reshape(L, -1, T, H, Dh) for t in (kq, vq, kp, vp)]
    live = np.ones((L, P), dtype=np.uint8)
    live[0, 7] = 0          # the exact copy's partner is dead in layer 0 only
    live[1, 2] = 0
    tau = 0.9
    r = oracle.match(dtype, mode, *a, live, tau, want_scores=True)
    S = brute_scores(*a, dtype, mode)
    assert np.allclose(r["scores"], S, atol=1e-12, rtol=0)
    Sl = np.where(live[:, None, :] == 1, S, -np.inf)
    assert np.array_equal(r["best_idx"], Sl.argmax(axis=2))
    assert np.allclose(r["best_score"], Sl.max(axis=2), atol=1e-12)
    assert np.allclose(r["second_score"], np.sort(Sl, axis=2)[:, :, -2], atol=1e-12)
    want_match = np.where(Sl.max(axis=2) >= tau, Sl.argmax(axis=2), -1)
    # keep the comparison away from rounding at the threshold
    assert (np.abs(Sl.max(axis=2) - tau) > 1e-9).all()
    assert np.array_equal(r["match_idx"], want_match)
    assert r["match_idx"][1, 1] == 7 and r["best_score"][1, 1] == 1.0
    assert r["best_idx"][0, 1] != 7        # dead blocks are skipped, not merely rejected
    # the pair-by-pair routine (used to sample full-size GPU results) must address layer, query and
    # pool block the same way: every triple, in a shuffled order, against the brute-force matrix
    li, qi, pi = [x.ravel().astype(np.int32) for x in np.meshgrid(np.arange(L), np.arange(Q), np.arange(P), indexing="ij")]
    order = rng.permutation(li.size)
    sp = oracle.score_pairs(dtype, mode, *a, li[order], qi[order], pi[order])
    assert np.allclose(sp, S[li[order], qi[order], pi[order]], atol=1e-12, rtol=0)


def test_tie_break_threshold_and_empty_pool(oracle):
    rng = np.random.RandomState(2)
    T, H, Dh = 2, 2, 4
    D = T * H * Dh
    pool = rng.randn(6, D)
    pool[4] = pool[1]                      # bit-identical pool blocks at 1 and 4
    q = pool[[4]]
    a = [blk(t, T, H, Dh, 0) for t in (q, q, pool, pool)]
    r = oracle.match(0, 0, *a, None, 1.0)
    assert r["best_idx"][0, 0] == 1 and r["match_idx"][0, 0] == 1        # lowest index; >= tau at tau = 1
    assert r["best_score"][0, 0] == 1.0 and r["second_score"][0, 0] == 1.0   # runner-up counted with multiplicity
    live = np.ones((1, 6), dtype=np.uint8)
    live[0, 1] = 0
    r = oracle.match(0, 0, *a, live, 1.0)
    assert r["best_idx"][0, 0] == 4
    r = oracle.match(0, 0, *a, np.zeros((1, 6), dtype=np.uint8), 0.5)
    assert r["best_idx"][0, 0] == -1 and r["match_idx"][0, 0] == -1 and r["best_score"][0, 0] == -np.inf
    r = oracle.match(0, 0, *a, None, np.nextafter(1.0, 2.0))
    assert r["match_idx"][0, 0] == -1 and r["best_idx"][0, 0] == 1


def test_cfg1_expected_matches(oracle):
    # Tiny workload: the 8 planted queries (sigma 0.1 -> score ~0.995) match their targets, the 24 fresh
    # ones (|score| ~ 1/sqrt(D)) match nothing.
    w = synth.WORKLOADS[1]
    pr = synth.make_problem(w, "cpu")
    plan = pr["plan"]
    r = oracle.match(0, w.mode, *(synth.bits(pr[n]) for n in ("kq", "vq", "kp", "vp")), pr["live"].numpy(), w.tau)
    want = np.full(w.Q, -1)
    want[plan.planted_slots] = plan.planted_targets
    assert np.array_equal(r["match_idx"][0], want)
    assert np.allclose(r["best_score"][0, plan.planted_slots], 1 / np.sqrt(1.01), atol=3e-3)
    fresh = np.setdiff1d(np.arange(w.Q), plan.planted_slots)
    assert (np.abs(r["best_score"][0, fresh]) < 0.06).all()


# ---------------------------------------------------------------- remap
def test_remap_golden(oracle):
    cases = json.load(open(os.path.join(GOLD, "remap_handworked.json")))["cases"]
    for c in cases:
        r = oracle.remap(np.array([c["tables"]], dtype=np.int32), c["query_ids"], c["pool_ids"],
                         np.array([c["match_idx"]], dtype=np.int32), c["P"], c["NB"],
                         np.array([c["refcount"]], dtype=np.int32))
        assert r["tables"][0].tolist() == c["tables_out"], c["name"]
        assert r["refcount"][0].tolist() == c["refcount_out"], c["name"]
        assert r["freed"][0].tolist() == c["freed"], c["name"]
        assert int(r["n_remapped"][0]) == c["n_remapped"], c["name"]


def random_remap_case(rng, L=3, P=40, Q=12, R=5, E=30):
    NB = P + Q + 4
    ids = rng.permutation(NB)
    pool_ids, query_ids = ids[:P].astype(np.int32), ids[P:P + Q].astype(np.int32)
    tables = rng.choice(np.concatenate([ids[:P + Q], [-1]]), size=(L, R, E)).astype(np.int32)
    refcount = np.stack([np.bincount(t[t >= 0], minlength=NB) for t in tables]).astype(np.int32)
    match = rng.randint(-1, P, size=(L, Q)).astype(np.int32)
    match[rng.rand(L, Q) < 0.4] = -1
    match[:, 1] = match[:, 0]              # two queries share a target
    return tables, query_ids, pool_ids, match, P, NB, refcount


def test_remap_invariants(oracle):
    rng = np.random.RandomState(8)
    for _ in range(10):
        tables, qids, pids, match, P, NB, rc = random_remap_case(rng)
        r = oracle.remap(tables, qids, pids, match, P, NB, rc)
        # references are conserved and refcounts stay equal to the number of table references
        assert np.array_equal(r["refcount"].sum(axis=1), rc.sum(axis=1))
        for l in range(tables.shape[0]):
            t = r["tables"][l]
            assert np.array_equal(r["refcount"][l], np.bincount(t[t >= 0], minlength=NB))
            matched = match[l] >= 0
            # every reference of a matched query block moved, so it is freed; unmatched ones are not
            assert np.array_equal(r["freed"][l].astype(bool), matched)
            assert not np.isin(t, qids[matched]).any()
            untouched = ~np.isin(tables[l], qids[matched])
            assert np.array_equal(t[untouched], tables[l][untouched])
            assert r["n_remapped"][l] == (~untouched).sum()
            # tables only point at blocks that are still referenced
            assert (r["refcount"][l][t[t >= 0]] >= 1).all()
        # idempotence: a second application changes nothing
        r2 = oracle.remap(r["tables"], qids, pids, match, P, NB, r["refcount"])
        assert np.array_equal(r2["tables"], r["tables"]) and np.array_equal(r2["refcount"], r["refcount"])
        assert (r2["n_remapped"] == 0).all()


def test_remap_no_match_is_identity(oracle):
    rng = np.random.RandomState(4)
    tables, qids, pids, match, P, NB, rc = random_remap_case(rng)
    match[:] = -1
    r = oracle.remap(tables, qids, pids, match, P, NB, rc)
    assert np.array_equal(r["tables"], tables) and np.array_equal(r["refcount"], rc)
    assert not r["freed"].any() and not r["n_remapped"].any()


# ---------------------------------------------------------------- candidate-restricted scoring
@pytest.mark.parametrize("mode", [0, 1])
def test_candidates_vs_exhaustive_and_brute_force(oracle, mode):
    # The candidate scores must be the entries of the brute-force score matrix at the listed indices,
    # and a list that names every live pool block must reproduce the exhaustive search.
    rng = np.random.RandomState(40 + mode)
    L, Q, P, T, H, Dh = 2, 4, 9, 2, 2, 4
    D = T * H * Dh
    kp, vp = rng.randn(L, P, D), rng.randn(L, P, D)
    kq, vq = rng.randn(L, Q, D), rng.randn(L, Q, D)
    kq[:, 0], vq[:, 0] = kp[:, 5], vp[:, 5]
    kp[:, 7], vp[:, 7] = kp[:, 5], vp[:, 5]          # bit-identical pool blocks: lowest index wins
    a = [enc(t, 0).reshape(L, -1, T, H, Dh) for t in (kq, vq, kp, vp)]
    live = np.ones((L, P), dtype=np.uint8)
    live[1, 5] = 0
    S = brute_scores(*a, 0, mode)
    cand = np.stack([np.stack([rng.permutation(P)[:4] for _ in range(Q)]) for _ in range(L)]).astype(np.int32)
    cand[:, 0, :] = [7, 2, 5, -1]
    cand[0, 1, 2] = P + 3                              # out of range: scores -inf
    r = oracle.candidates(0, mode, *a, cand, live, 0.9)
    for l in range(L):
        for q in range(Q):
            for c in range(4):
                p = cand[l, q, c]
                ok = 0 <= p < P and live[l, p]
                if ok:
                    assert r["scores"][l, q, c] == pytest.approx(S[l, q, p], abs=1e-12)
                else:
                    assert r["scores"][l, q, c] == -np.inf
    assert r["best_idx"][0, 0] == 5 and r["match_idx"][0, 0] == 5 and r["best_score"][0, 0] == 1.0
    assert r["best_idx"][1, 0] == 7                    # 5 is dead in layer 1
    assert oracle.candidates(0, mode, *a, cand, live, 1.0)["match_idx"][0, 0] == 5      # inclusive threshold
    full = np.tile(np.arange(P, dtype=np.int32), (L, Q, 1))
    rf = oracle.candidates(0, mode, *a, full, live, 0.9)
    rm = oracle.match(0, mode, *a, live, 0.9)
    assert np.array_equal(rf["best_idx"], rm["best_idx"]) and np.array_equal(rf["match_idx"], rm["match_idx"])
    assert np.allclose(rf["best_score"], rm["best_score"], atol=1e-12)
    empty = oracle.candidates(0, mode, *a, np.full((L, Q, 2), -1, np.int32), live, 0.9)
    assert (empty["best_idx"] == -1).all() and np.isneginf(empty["best_score"]).all()


# ---- the paper's own measure: layer-mean Euclidean block distance (Sec. IV-A Stage 2, block-distance equation)

def layers(rows, T, H, Dh, dtype):
    """[L][D] floats -> [L][1][T][H][Dh] bits (one block per layer)."""
    return enc(np.asarray(rows, dtype=np.float32), dtype).reshape(len(rows), 1, T, H, Dh)


@pytest.mark.parametrize("dtype", [0, 1])
def test_layer_mean_golden(oracle, dtype):
    cases = json.load(open(os.path.join(GOLD, "layer_mean_handworked.json")))["cases"]
    for c in cases:
        a = [layers(c[n], c["T"], c["H"], c["Dh"], dtype) for n in ("kq", "vq", "kp", "vp")]
        r = oracle.layer_mean(dtype, *a, None, 1e9, want_dist=True)
        assert r["dist"][0, 0] == pytest.approx(c["dist"], abs=1e-13), c["name"]
        assert r["best_dist"][0] == pytest.approx(c["dist"], abs=1e-13) and r["best_idx"][0] == 0


def rand_kv(rng, L, n, T, H, Dh, dtype):
    return enc(rng.randn(L, n, T, H, Dh), dtype)


@pytest.mark.parametrize("dtype", [0, 1])
def test_layer_mean_vs_library_norm_and_expansion(oracle, dtype):
    rng = np.random.RandomState(5)
    L, Q, P, T, H, Dh = 3, 4, 7, 2, 3, 8
    kq, vq, kp, vp = (rand_kv(rng, L, n, T, H, Dh, dtype) for n in (Q, Q, P, P))
    r = oracle.layer_mean(dtype, kq, vq, kp, vp, None, 0.0, want_dist=True)
    # (1) numpy's norm routine on library-decoded values
    f = [dec(x, dtype).reshape(L, -1, T * H * Dh) for x in (kq, vq, kp, vp)]
    want = np.zeros((Q, P))
    for l in range(L):
        for q in range(Q):
            for p in range(P):
                want[q, p] += (np.linalg.norm(f[0][l, q] - f[2][l, p]) + np.linalg.norm(f[1][l, q] - f[3][l, p])) / (2 * T * H)
    want /= L
    assert np.allclose(r["dist"], want, rtol=1e-13, atol=0)
    # (2) the expansion of Stage 2 through the separately pinned norms and cosine scores:
    #     with V := K the score is cos(Kq, Kp), so |x-y|^2 = |x|^2 + |y|^2 - 2 cos sqrt(|x|^2 |y|^2)
    nq, _ = oracle.block_norms(dtype, oracle.BLOCK, kq, kq)
    npk, _ = oracle.block_norms(dtype, oracle.BLOCK, kp, kp)
    cosk = oracle.match(dtype, oracle.BLOCK, kq, kq, kp, kp, None, 0.0, want_scores=True)["scores"]
    rk = oracle.layer_mean(dtype, kq, kq, kp, kp, None, 0.0, want_dist=True)["dist"]   # = mean_l 2 dK / (2dh)
    dk = np.sqrt(nq[:, :, None] + npk[:, None, :] - 2 * cosk * np.sqrt(nq[:, :, None] * npk[:, None, :]))
    assert np.allclose(rk, (2 * dk / (2 * T * H)).mean(axis=0), rtol=1e-11)
    # (3) the direct single-pair routine
    for (l, q, p) in [(0, 0, 0), (2, 3, 6)]:
        one = oracle.layer_mean(dtype, kq[l:l + 1, q:q + 1], vq[l:l + 1, q:q + 1], kp[l:l + 1, p:p + 1], vp[l:l + 1, p:p + 1],
                                None, 0.0, want_dist=True)["dist"][0, 0]
        sk = oracle.sqdist(dtype, kq[l, q].ravel(), kp[l, p].ravel())
        sv = oracle.sqdist(dtype, vq[l, q].ravel(), vp[l, p].ravel())
        assert one == pytest.approx((np.sqrt(sk) + np.sqrt(sv)) / (2 * T * H), rel=1e-14)


def test_layer_mean_metric_properties(oracle):
    rng = np.random.RandomState(8)
    L, n, T, H, Dh = 2, 5, 2, 2, 4
    k, v = rand_kv(rng, L, n, T, H, Dh, 0), rand_kv(rng, L, n, T, H, Dh, 0)
    d = oracle.layer_mean(0, k, v, k, v, None, 0.0, want_dist=True)["dist"]
    assert (np.diag(d) == 0).all()                         # identity
    assert np.array_equal(d, d.T)                          # symmetry (same products, same order)
    for a in range(n):                                     # triangle inequality (sums of norms are norms of a product space)
        for b in range(n):
            for c in range(n):
                assert d[a, c] <= d[a, b] + d[b, c] + 1e-12
    # doubling every value (exact in fp16) doubles the distance
    k2 = enc(2 * dec(k, 0), 0).reshape(k.shape)
    v2 = enc(2 * dec(v, 0), 0).reshape(v.shape)
    d2 = oracle.layer_mean(0, k2, v2, k2, v2, None, 0.0, want_dist=True)["dist"]
    assert np.allclose(d2, 2 * d, rtol=1e-14)
    # the mean over layers: identical layers give the single-layer value, the layer order is irrelevant,
    # and the two-layer value is the average of the single-layer values
    d0 = oracle.layer_mean(0, k[:1], v[:1], k[:1], v[:1], None, 0.0, want_dist=True)["dist"]
    d1 = oracle.layer_mean(0, k[1:], v[1:], k[1:], v[1:], None, 0.0, want_dist=True)["dist"]
    rep = oracle.layer_mean(0, np.repeat(k[:1], 3, 0), np.repeat(v[:1], 3, 0), np.repeat(k[:1], 3, 0), np.repeat(v[:1], 3, 0),
                            None, 0.0, want_dist=True)["dist"]
    assert np.allclose(rep, d0, rtol=1e-14)
    assert np.allclose(d, 0.5 * (d0 + d1), rtol=1e-14)
    flip = oracle.layer_mean(0, k[::-1], v[::-1], k[::-1], v[::-1], None, 0.0, want_dist=True)["dist"]
    assert np.allclose(flip, d, rtol=1e-14)
    # K and V enter symmetrically
    sw = oracle.layer_mean(0, v, k, v, k, None, 0.0, want_dist=True)["dist"]
    assert np.allclose(sw, d, rtol=1e-14)


def test_layer_mean_selection_rules(oracle):
    T, H, Dh = 1, 1, 4
    mk = lambda rows: enc(np.asarray(rows, dtype=np.float32), 0).reshape(1, len(rows), T, H, Dh)
    kq = mk([[0, 0, 0, 0], [10, 0, 0, 0]])
    vq = mk([[0, 0, 0, 0], [0, 0, 0, 0]])
    kp = mk([[4, 0, 0, 0], [0, 2, 0, 0], [0, 0, 2, 0], [0, 0, 0, 6], [10, 0, 0, 0]])
    vp = mk([[0, 0, 0, 0]] * 5)
    # query 0: distances 2, 1, 1, 3, 5 -> tie between pool 1 and 2 goes to 1, runner-up is the other 1
    r = oracle.layer_mean(0, kq, vq, kp, vp, None, 1.0, want_dist=True)
    assert np.allclose(r["dist"][0], [2, 1, 1, 3, 5])
    assert r["best_idx"].tolist() == [1, 4] and r["best_dist"].tolist() == [1.0, 0.0]
    assert r["second_dist"][0] == 1.0 and r["second_dist"][1] == 3.0   # query 1: |10 - 4| / 2
    assert r["match_idx"].tolist() == [1, 4]               # distance == threshold still matches
    assert oracle.layer_mean(0, kq, vq, kp, vp, None, 0.999)["match_idx"].tolist() == [-1, 4]
    # dead blocks are skipped by the search, not rejected after it
    live = np.array([1, 0, 1, 1, 0], dtype=np.uint8)
    r = oracle.layer_mean(0, kq, vq, kp, vp, live, 1.0)
    assert r["best_idx"].tolist() == [2, 0] and r["match_idx"].tolist() == [2, -1]
    assert r["best_dist"][1] == 3.0 and r["second_dist"][0] == 2.0
    # nothing live / empty pool
    r = oracle.layer_mean(0, kq, vq, kp, vp, np.zeros(5, np.uint8), 1e9)
    assert r["best_idx"].tolist() == [-1, -1] and np.isposinf(r["best_dist"]).all() and r["match_idx"].tolist() == [-1, -1]
    r = oracle.layer_mean(0, kq, vq, kp[:, :0], vp[:, :0], None, 1e9)
    assert r["best_idx"].tolist() == [-1, -1] and np.isposinf(r["second_dist"]).all()


def test_layer_mean_noisy_copy_law(oracle):
    # a copy with N(0, sigma^2) noise on every element sits at about 2 sigma sqrt(D) / (2dh) = sigma sqrt(Dh/(d h)) ... per tensor,
    # i.e. d = sigma * sqrt(Dh / (T H)) for K plus V; fresh blocks at sqrt(2) times that with sigma = 1
    w = synth.scaled(synth.WORKLOADS[1], L=2, P=24, Q=8, E=24, planted_frac=0.5, sigma=0.1)
    pr = synth.make_problem(w, "cpu")
    plan = pr["plan"]
    r = oracle.layer_mean(0, *(synth.bits(pr[n]) for n in ("kq", "vq", "kp", "vp")), None, 0.5, want_dist=True)
    unit = np.sqrt(w.Dh / (w.T * w.H))
    d_planted = r["dist"][plan.planted_slots, plan.planted_targets]
    assert np.allclose(d_planted, w.sigma * unit, rtol=0.03)
    fresh = np.setdiff1d(np.arange(w.Q), plan.planted_slots)
    assert np.allclose(r["dist"][fresh], np.sqrt(2) * unit, rtol=0.05)
    assert (r["match_idx"][plan.planted_slots] == plan.planted_targets).all() and (r["match_idx"][fresh] == -1).all()


# ---- percentile-based adaptive threshold (Sec. IV-A, PAT; p = 80 in the evaluation's parameter paragraph)

def test_pat_hand_cases(oracle):
    s = np.array([5, 1, 4, 2, 3], dtype=np.float32)
    # nearest rank on 5 samples: k = ceil(p/100 * 5)
    for p, want in ((80, 4), (100, 5), (20, 1), (50, 3), (60, 3), (61, 4), (0, 1), (1, 1)):
        thr, n = oracle.pat_threshold(s, p)
        assert (thr, n) == (want, 5), p
    # p = 100 accepts every collected distance, smaller p accepts at least p % of them
    thr, _ = oracle.pat_threshold(s, 100)
    assert (s <= thr).all()
    # samples without a candidate (+inf), NaN and -inf are left out
    thr, n = oracle.pat_threshold(np.array([np.inf, 2, np.nan, 1, -np.inf, 3], dtype=np.float32), 100)
    assert (thr, n) == (3, 3)
    thr, n = oracle.pat_threshold(np.array([np.inf, np.inf], dtype=np.float32), 80)
    assert np.isneginf(thr) and n == 0
    thr, n = oracle.pat_threshold(np.zeros(0, dtype=np.float32), 80)
    assert np.isneginf(thr) and n == 0
    # duplicates and a single sample
    assert oracle.pat_threshold(np.array([2, 2, 2, 7], dtype=np.float32), 75)[0] == 2
    assert oracle.pat_threshold(np.array([2, 2, 2, 7], dtype=np.float32), 76)[0] == 7
    assert oracle.pat_threshold(np.array([9], dtype=np.float32), 0)[0] == 9
    # the rank is formed from the double the caller passes: 0.1 % of 1000 samples is exactly one sample (the smallest);
    # the same percentile rounded to float first (0.100000001...) would reach the second
    s1000 = np.arange(1000, dtype=np.float32)[::-1].copy()
    assert oracle.pat_threshold(s1000, 0.1)[0] == 0
    assert oracle.pat_threshold(s1000, 0.2)[0] == 1


def test_pat_vs_library_quantile_and_definition(oracle):
    rng = np.random.RandomState(21)
    for n in (1, 2, 7, 100, 1001, 4096):
        s = np.abs(rng.randn(n)).astype(np.float32)
        s[rng.rand(n) < 0.1] = s[0]                     # ties
        for p in (0.0, 20.0, 50.0, 80.0, 99.9, 100.0, 33.3):
            thr, cnt = oracle.pat_threshold(s, p)
            assert cnt == n
            # numpy's nearest-rank quantile (inverse of the empirical distribution function)
            assert thr == np.percentile(s, p, method="inverted_cdf"), (n, p)
            # the two inequalities that define a p-quantile of a sample
            assert (s <= thr).sum() >= np.ceil(p / 100 * n - 1e-9)
            assert (s < thr).sum() <= p / 100 * n + 1e-9
    # order of the samples is irrelevant; negative values sort below positive ones
    s = rng.randn(500).astype(np.float32)
    assert oracle.pat_threshold(s, 80)[0] == oracle.pat_threshold(s[::-1], 80)[0] == np.sort(s)[399]


def test_apply_threshold(oracle):
    idx = np.array([3, -1, 5, 7, 2], dtype=np.int32)
    d = np.array([0.5, np.inf, 0.25, 0.75, np.nan], dtype=np.float32)
    assert oracle.apply_threshold(idx, d, np.float32(0.5)).tolist() == [3, -1, 5, -1, -1]   # inclusive; NaN never matches
    assert oracle.apply_threshold(idx, d, np.float32(-np.inf)).tolist() == [-1] * 5          # warm-up: reuse disabled
    assert oracle.apply_threshold(idx, d, np.float32(np.inf)).tolist() == [3, -1, 5, 7, -1]


# ---- streaming pool maintenance (Sec. IV-B: the search is part of every decoding step)

def test_pool_admit_hand_case(oracle):
    T, H, Dh, L = 1, 1, 2, 2
    kq = np.arange(100, 100 + L * 4 * 2, dtype=np.uint16).reshape(L, 4, T, H, Dh)
    vq = kq + 50
    kp = np.arange(L * 5 * 2, dtype=np.uint16).reshape(L, 5, T, H, Dh)
    vp = kp + 20
    kp0, vp0 = kp.copy(), vp.copy()
    qn = np.arange(L * 4, dtype=np.float64).reshape(L, 4) + 0.5
    pn = -np.ones((L, 5))
    pk, pv = pn.copy(), pn.copy()
    live = np.array([1, 0, 1, 0, 0], dtype=np.uint8)
    slot, n = oracle.pool_admit(kq, vq, qn, qn + 100, kp, vp, pk, pv, live, np.array([-1, 3, -1, -1], dtype=np.int32))
    # unmatched queries 0, 2, 3 take the dead slots 1, 3, 4 in that order; query 1 is matched and needs none
    assert slot.tolist() == [1, -1, 3, 4] and n == 3 and live.tolist() == [1, 1, 1, 1, 1]
    for q, s in ((0, 1), (2, 3), (3, 4)):
        assert np.array_equal(kp[:, s], kq[:, q]) and np.array_equal(vp[:, s], vq[:, q])
        assert np.array_equal(pk[:, s], qn[:, q]) and np.array_equal(pv[:, s], qn[:, q] + 100)
    for s in (0, 2):                                   # live slots are untouched
        assert np.array_equal(kp[:, s], kp0[:, s]) and np.array_equal(vp[:, s], vp0[:, s]) and (pk[:, s] == -1).all()


def test_pool_admit_full_pool_and_noop(oracle):
    rng = np.random.RandomState(12)
    L, Q, P, T, H, Dh = 2, 6, 7, 1, 2, 4
    kq, vq = (rng.randint(0, 60000, (L, Q, T, H, Dh)).astype(np.uint16) for _ in range(2))
    kp, vp = (rng.randint(0, 60000, (L, P, T, H, Dh)).astype(np.uint16) for _ in range(2))
    qk, qv = rng.rand(L, Q, H), rng.rand(L, Q, H)       # per-head norm layout
    pk, pv = rng.rand(L, P, H), rng.rand(L, P, H)
    live = np.array([1, 1, 0, 1, 1, 0, 1], dtype=np.uint8)
    before = int(live.sum())
    m = np.array([-1, -1, 2, -1, -1, -1], dtype=np.int32)
    slot, n = oracle.pool_admit(kq, vq, qk, qv, kp, vp, pk, pv, live, m)
    # two free slots for five unmatched queries: the first two in order get them, the rest are left out
    assert slot.tolist() == [2, 5, -1, -1, -1, -1] and n == 2 and int(live.sum()) == before + n
    assert np.array_equal(pk[:, 2], qk[:, 0]) and np.array_equal(pv[:, 5], qv[:, 1])
    # a second call finds no room and changes nothing; so does a call in which every query matched
    snap = [a.copy() for a in (kp, vp, pk, pv, live)]
    slot, n = oracle.pool_admit(kq, vq, qk, qv, kp, vp, pk, pv, live, m)
    assert n == 0 and (slot == -1).all() and all(np.array_equal(a, b) for a, b in zip(snap, (kp, vp, pk, pv, live)))
    live[3] = 0
    slot, n = oracle.pool_admit(kq, vq, qk, qv, kp, vp, pk, pv, live, np.zeros(Q, dtype=np.int32))
    assert n == 0 and live[3] == 0


def test_pool_admit_closes_the_loop(oracle):
    # a block admitted in one step is found as an exact partner (distance 0, score 1) by its copy in the next step
    w = synth.scaled(synth.WORKLOADS[1], L=2, P=12, Q=4, E=12, planted_frac=0.0)
    pr = synth.make_problem(w, "cpu")
    a = {n: synth.bits(pr[n]).copy() for n in ("kq", "vq", "kp", "vp")}
    live = np.ones(w.P, dtype=np.uint8)
    live[[5, 9]] = 0
    qk, qv = oracle.block_norms(0, oracle.BLOCK, a["kq"], a["vq"])
    pk, pv = oracle.block_norms(0, oracle.BLOCK, a["kp"], a["vp"])
    first = oracle.layer_mean(0, a["kq"], a["vq"], a["kp"], a["vp"], live, 0.5)
    assert (first["match_idx"] == -1).all()
    slot, n = oracle.pool_admit(a["kq"], a["vq"], qk, qv, a["kp"], a["vp"], pk, pv, live, first["match_idx"])
    assert slot.tolist() == [5, 9, -1, -1] and n == 2
    # the cached norms that travelled with the blocks are the norms of what now sits in the slots
    pk2, pv2 = oracle.block_norms(0, oracle.BLOCK, a["kp"], a["vp"])
    assert np.array_equal(pk, pk2) and np.array_equal(pv, pv2)
    again = oracle.layer_mean(0, a["kq"], a["vq"], a["kp"], a["vp"], live, 0.5)
    assert again["best_idx"][:2].tolist() == [5, 9] and (again["best_dist"][:2] == 0).all()
    assert again["match_idx"].tolist() == [5, 9, -1, -1]
    s = oracle.match(0, oracle.BLOCK, a["kq"], a["vq"], a["kp"], a["vp"], np.tile(live, (w.L, 1)), 0.95)
    assert (s["best_score"][:, :2] == 1.0).all() and (s["match_idx"][:, :2] == np.array([5, 9])).all()


# ---- Stage 2 as the paper runs it: layer-mean distance of listed candidate pairs

def test_candidate_distances_vs_matrix_and_rules(oracle):
    rng = np.random.RandomState(31)
    L, Q, P, T, H, Dh = 3, 5, 9, 2, 2, 8
    kq, vq, kp, vp = (rand_kv(rng, L, n, T, H, Dh, 0) for n in (Q, Q, P, P))
    live = np.ones(P, dtype=np.uint8)
    live[4] = 0
    full = oracle.layer_mean(0, kq, vq, kp, vp, None, 0.0, want_dist=True)["dist"]      # pinned separately
    cand = rng.randint(0, P, size=(Q, 6)).astype(np.int32)
    cand[:, 1] = -1                       # empty slot
    cand[0, 0] = P + 3                    # out of range
    cand[1, 2] = 4                        # dead
    cand[2, 3] = cand[2, 4]               # listed twice
    cand[3, :] = -1                       # empty list
    r = oracle.candidate_distances(0, kq, vq, kp, vp, cand, live, 1e9)
    for q in range(Q):
        for c in range(6):
            p = cand[q, c]
            if p < 0 or p >= P or not live[p]:
                assert np.isposinf(r["dist"][q, c])
            else:
                assert r["dist"][q, c] == pytest.approx(full[q, p], rel=1e-14)
    assert r["best_idx"][3] == -1 and np.isposinf(r["best_dist"][3]) and r["match_idx"][3] == -1
    for q in (0, 1, 2, 4):
        valid = [(full[q, p], p) for p in cand[q] if 0 <= p < P and live[p]]
        assert (r["best_dist"][q], r["best_idx"][q]) == pytest.approx(min(valid))
    # the hand-worked two-layer case through a list
    c = json.load(open(os.path.join(GOLD, "layer_mean_handworked.json")))["cases"][1]
    a = [layers(c[n], c["T"], c["H"], c["Dh"], 0) for n in ("kq", "vq", "kp", "vp")]
    r = oracle.candidate_distances(0, *a, np.array([[0, -1, 0]], dtype=np.int32), None, 4.5)
    assert r["dist"][0].tolist() == [4.5, np.inf, 4.5] and r["match_idx"][0] == 0          # inclusive threshold
    assert oracle.candidate_distances(0, *a, np.array([[0]], dtype=np.int32), None, 4.49)["match_idx"][0] == -1
    # ties go to the lowest pool index whatever the order in the list
    kp2 = np.concatenate([kp[:, :1]] * 3, axis=1)
    vp2 = np.concatenate([vp[:, :1]] * 3, axis=1)
    for order in ([2, 1, 0], [1, 0, 2], [0, 2, 1]):
        r = oracle.candidate_distances(0, kq, vq, kp2, vp2, np.tile(np.array([order], dtype=np.int32), (Q, 1)), None, 1e9)
        assert (r["best_idx"] == 0).all(), order


# ---- pool metadata and eviction (Sec. IV-B: free at reference count 0; Sec. IV-A: LRU order on block metadata)

def test_pool_touch_and_release_hand_cases(oracle):
    stamp = np.array([5, 5, 5, 5, 5], dtype=np.int32)
    oracle.pool_touch(np.array([3, -1, 0, 7, 3], dtype=np.int32), 9, stamp)      # -1 and 7 are outside: skipped
    assert stamp.tolist() == [9, 5, 5, 9, 5]
    rc = np.array([2, 1, 0, 3], dtype=np.int32)
    oracle.refcount_release(np.array([0, 3, 3, -1, 9, 0], dtype=np.int32), rc)   # with multiplicity
    assert rc.tolist() == [0, 1, 0, 1]


def test_pool_evict_hand_cases(oracle):
    U = np.array([-1, -1, -1], dtype=np.int32)          # three unmatched queries
    # slots:            0  1  2  3  4  5
    live = np.array([1, 1, 0, 1, 1, 1], dtype=np.uint8)
    refc = np.array([0, 2, 0, 0, 0, 1], dtype=np.int32)
    used = np.array([7, 1, 0, 4, 4, 0], dtype=np.int32)
    # one slot is free already; two more are needed: the unreferenced ones are 0, 3, 4 with stamps 7, 4, 4:
    # slots 3 and 4 go (stamp 4 before 7); slot 1 (stamp 1) and slot 5 (stamp 0) are referenced and stay
    lv = live.copy()
    assert oracle.pool_evict(lv, refc, used, U) == (3, 2)
    assert lv.tolist() == [1, 1, 0, 0, 0, 1]
    # one more needed than there are candidates: all three unreferenced slots go, and that is all
    lv = live.copy()
    assert oracle.pool_evict(lv, refc, used, U, extra_wanted=2) == (4, 3)
    assert lv.tolist() == [0, 1, 0, 0, 0, 1]
    # ties go to the lowest slot: only one of the two stamp-4 slots is needed
    lv = live.copy()
    assert oracle.pool_evict(lv, refc, used, np.array([-1, 5, -1], dtype=np.int32)) == (2, 1)
    assert lv.tolist() == [1, 1, 0, 0, 1, 1]
    # without reference counts every live slot is a candidate: stamps 0 (slot 5), 1 (slot 1) go first
    lv = live.copy()
    assert oracle.pool_evict(lv, None, used, U) == (3, 2)
    assert lv.tolist() == [1, 0, 0, 1, 1, 0]
    # enough room already, or nothing unmatched: untouched
    lv = live.copy()
    assert oracle.pool_evict(lv, refc, used, np.array([-1, 2], dtype=np.int32)) == (1, 0) and np.array_equal(lv, live)
    assert oracle.pool_evict(lv, refc, used, np.array([0, 2], dtype=np.int32)) == (1, 0) and np.array_equal(lv, live)
    # empty pool
    assert oracle.pool_evict(np.zeros(0, np.uint8), None, np.zeros(0, np.int32), U) == (0, 0)


def test_pool_evict_vs_sorting_and_invariants(oracle):
    rng = np.random.RandomState(31)
    for case in range(40):
        P = int(rng.choice([1, 2, 17, 64, 300, 1500]))
        live = (rng.rand(P) < rng.choice([0.5, 0.9, 1.0])).astype(np.uint8)
        refc = (rng.randint(0, 3, P) * (rng.rand(P) < 0.6)).astype(np.int32)
        used = rng.randint(0, rng.choice([2, 5, 1000]), P).astype(np.int32)     # few distinct stamps: many ties
        m = np.where(rng.rand(int(rng.randint(0, 2 * P + 2))) < 0.6, -1, 0).astype(np.int32)
        extra = int(rng.randint(0, 3))
        use_rc = rng.rand() < 0.7
        lv = live.copy()
        n_free, n_ev = oracle.pool_evict(lv, refc if use_rc else None, used, m, extra)
        # the same by sorting the candidates by (stamp, slot), written with a library sort
        wanted = int((m < 0).sum()) + extra
        free0 = int((live == 0).sum())
        cand = np.flatnonzero((live == 1) & ((refc == 0) if use_rc else True))
        order = cand[np.lexsort((cand, used[cand]))]
        k = min(max(wanted - free0, 0), order.size)
        want = live.copy()
        want[order[:k]] = 0
        assert np.array_equal(lv, want), case
        assert (n_free, n_ev) == (free0 + k, k)
        # invariants: nothing referenced left, nothing dead came back, survivors are not older than victims
        gone = np.flatnonzero((live == 1) & (lv == 0))
        if use_rc:
            assert (refc[gone] == 0).all()
        assert (lv <= live).all()
        stay = np.setdiff1d(cand, gone)
        if gone.size and stay.size:
            assert used[gone].max() <= used[stay].min()
