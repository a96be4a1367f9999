"""ctypes front end of the CPU oracle (``rc_oracle.c``).

TEST INFRASTRUCTURE, not product code: only ``tests/``, the smoke check and the
CPU-baseline leg of ``bench.py`` may import this module.  It shares nothing with
the HIP path and never imports it.

KV tensors are passed as numpy ``uint16`` arrays holding the raw fp16 / bf16 bit
patterns, shaped ``[L][n][T][H][Dh]`` and C-contiguous.  All results are double
precision / int32 numpy arrays.  What each function computes, and the passages
of the paper it follows, is stated in ``rc_oracle.c``.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rc_oracle.c")
# RC_ORACLE_LIB names another build of the oracle to load instead (the tests use it to show that
# the pins reject copies of rc_oracle.c with a planted mistake); such a library is never rebuilt here.
_OVERRIDE = os.environ.get("RC_ORACLE_LIB")
_LIB = _OVERRIDE or os.path.join(_HERE, "librc_oracle.so")

F16, BF16 = 0, 1
BLOCK, PER_HEAD_ALL = 0, 1

_lib = None


def build(force=False):
    """Compile the oracle with gcc (plain -O2, OpenMP over independent blocks)."""
    if _OVERRIDE:
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _kv(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16 and a.ndim == 5, "KV must be uint16 bits shaped [L][n][T][H][Dh]"
    return a


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def n_threads():
    """OpenMP threads the oracle's parallel loops will use."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        return int(env.split(",")[0])
    return len(os.sched_getaffinity(0))


def decode(dtype, bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float64)
    _check(_load().rc_oracle_decode(ctypes.c_int(dtype), _p(bits), ctypes.c_int64(bits.size), _p(out)), "decode")
    return out


def block_norms(dtype, mode, k, v):
    """Squared norms -> (ksq, vsq), each [L][n] (BLOCK) or [L][n][H] (PER_HEAD_ALL)."""
    k, v = _kv(k), _kv(v)
    assert k.shape == v.shape
    L, n, T, H, Dh = k.shape
    shape = (L, n) if mode == BLOCK else (L, n, H)
    ksq = np.zeros(shape, dtype=np.float64)
    vsq = np.zeros(shape, dtype=np.float64)
    rc = _load().rc_oracle_block_norms(
        ctypes.c_int(dtype), ctypes.c_int(mode), ctypes.c_int(L), ctypes.c_int(T), ctypes.c_int(H),
        ctypes.c_int(Dh), ctypes.c_int64(n * T * H * Dh), _p(k), _p(v), ctypes.c_int64(n), _p(ksq), _p(vsq))
    _check(rc, "block_norms")
    return ksq, vsq


def sqdist(dtype, x, y):
    """Sum of (x-y)^2 over two equally sized bit arrays, by subtracting and squaring."""
    x = np.ascontiguousarray(x, dtype=np.uint16).ravel()
    y = np.ascontiguousarray(y, dtype=np.uint16).ravel()
    assert x.size == y.size
    out = ctypes.c_double(0.0)
    _check(_load().rc_oracle_sqdist(ctypes.c_int(dtype), _p(x), _p(y), ctypes.c_int64(x.size), ctypes.byref(out)),
           "sqdist")
    return out.value


def score_pairs(dtype, mode, kq, vq, kp, vp, li, qi, pi):
    """Scores of the listed (layer, query, pool) triples, each computed from scratch."""
    kq, vq, kp, vp = _kv(kq), _kv(vq), _kv(kp), _kv(vp)
    L, Q, T, H, Dh = kq.shape
    P = kp.shape[1]
    li = np.ascontiguousarray(li, dtype=np.int32)
    qi = np.ascontiguousarray(qi, dtype=np.int32)
    pi = np.ascontiguousarray(pi, dtype=np.int32)
    assert li.shape == qi.shape == pi.shape
    assert (li >= 0).all() and (li < L).all() and (qi >= 0).all() and (qi < Q).all()
    assert (pi >= 0).all() and (pi < P).all()
    out = np.zeros(li.shape, dtype=np.float64)
    D = T * H * Dh
    rc = _load().rc_oracle_score_pairs(
        ctypes.c_int(dtype), ctypes.c_int(mode), ctypes.c_int(T), ctypes.c_int(H), ctypes.c_int(Dh),
        _p(kq), _p(vq), ctypes.c_int64(Q * D), _p(kp), _p(vp), ctypes.c_int64(P * D),
        ctypes.c_int64(li.size), _p(li), _p(qi), _p(pi), _p(out))
    _check(rc, "score_pairs")
    return out


def match(dtype, mode, kq, vq, kp, vp, live, tau, want_scores=False):
    """Exhaustive search.  Returns dict(best_idx, best_score, match_idx, second_score[, scores])."""
    kq, vq, kp, vp = _kv(kq), _kv(vq), _kv(kp), _kv(vp)
    L, Q, T, H, Dh = kq.shape
    P = kp.shape[1]
    assert vq.shape == kq.shape and vp.shape == kp.shape and kp.shape[0] == L and kp.shape[2:] == kq.shape[2:]
    if live is not None:
        live = np.ascontiguousarray(live, dtype=np.uint8)
        assert live.shape == (L, P)
    D = T * H * Dh
    best_idx = np.zeros((L, Q), dtype=np.int32)
    match_idx = np.zeros((L, Q), dtype=np.int32)
    best_score = np.zeros((L, Q), dtype=np.float64)
    second = np.zeros((L, Q), dtype=np.float64)
    scores = np.zeros((L, Q, P), dtype=np.float64) if want_scores else None
    rc = _load().rc_oracle_match(
        ctypes.c_int(dtype), ctypes.c_int(mode), ctypes.c_int(L), ctypes.c_int(T), ctypes.c_int(H), ctypes.c_int(Dh),
        _p(kq), _p(vq), ctypes.c_int64(Q * D), ctypes.c_int64(Q),
        _p(kp), _p(vp), ctypes.c_int64(P * D), ctypes.c_int64(P),
        _p(live), ctypes.c_double(tau),
        _p(best_idx), _p(best_score), _p(match_idx), _p(second), _p(scores))
    _check(rc, "match")
    out = dict(best_idx=best_idx, best_score=best_score, match_idx=match_idx, second_score=second)
    if want_scores:
        out["scores"] = scores
    return out


def candidates(dtype, mode, kq, vq, kp, vp, cand, live, tau):
    """Scores of the listed candidates [L][Q][C] (pool index or -1) and the best of each list."""
    kq, vq, kp, vp = _kv(kq), _kv(vq), _kv(kp), _kv(vp)
    L, Q, T, H, Dh = kq.shape
    P = kp.shape[1]
    cand = np.ascontiguousarray(cand, dtype=np.int32)
    assert cand.ndim == 3 and cand.shape[:2] == (L, Q)
    C = cand.shape[2]
    if live is not None:
        live = np.ascontiguousarray(live, dtype=np.uint8)
        assert live.shape == (L, P)
    D = T * H * Dh
    scores = np.zeros((L, Q, C), dtype=np.float64)
    best_idx = np.zeros((L, Q), dtype=np.int32)
    match_idx = np.zeros((L, Q), dtype=np.int32)
    best_score = np.zeros((L, Q), dtype=np.float64)
    rc = _load().rc_oracle_candidates(
        ctypes.c_int(dtype), ctypes.c_int(mode), ctypes.c_int(L), ctypes.c_int(T), ctypes.c_int(H), ctypes.c_int(Dh),
        _p(kq), _p(vq), ctypes.c_int64(Q * D), ctypes.c_int64(Q), _p(kp), _p(vp), ctypes.c_int64(P * D),
        ctypes.c_int64(P), _p(cand), ctypes.c_int64(C), _p(live), ctypes.c_double(tau),
        _p(scores), _p(best_idx), _p(best_score), _p(match_idx))
    _check(rc, "candidates")
    return dict(scores=scores, best_idx=best_idx, best_score=best_score, match_idx=match_idx)


def layer_mean(dtype, kq, vq, kp, vp, live, thr, want_dist=False):
    """Layer-mean block distance and the per-block decision.  live is [P] or None.

    Returns dict(best_idx, best_dist, match_idx, second_dist[, dist]) with [Q] arrays (dist is [Q][P])."""
    kq, vq, kp, vp = _kv(kq), _kv(vq), _kv(kp), _kv(vp)
    L, Q, T, H, Dh = kq.shape
    P = kp.shape[1]
    assert vq.shape == kq.shape and vp.shape == kp.shape and kp.shape[0] == L and kp.shape[2:] == kq.shape[2:]
    if live is not None:
        live = np.ascontiguousarray(live, dtype=np.uint8)
        assert live.shape == (P,)
    D = T * H * Dh
    best_idx = np.zeros(Q, dtype=np.int32)
    match_idx = np.zeros(Q, dtype=np.int32)
    best = np.zeros(Q, dtype=np.float64)
    second = np.zeros(Q, dtype=np.float64)
    dist = np.zeros((Q, P), dtype=np.float64) if want_dist else None
    rc = _load().rc_oracle_layer_mean(
        ctypes.c_int(dtype), ctypes.c_int(L), ctypes.c_int(T), ctypes.c_int(H), ctypes.c_int(Dh),
        _p(kq), _p(vq), ctypes.c_int64(Q * D), ctypes.c_int64(Q),
        _p(kp), _p(vp), ctypes.c_int64(P * D), ctypes.c_int64(P),
        _p(live), ctypes.c_double(thr),
        _p(best_idx), _p(best), _p(match_idx), _p(second), _p(dist))
    _check(rc, "layer_mean")
    out = dict(best_idx=best_idx, best_dist=best, match_idx=match_idx, second_dist=second)
    if want_dist:
        out["dist"] = dist
    return out


def candidate_distances(dtype, kq, vq, kp, vp, cand, live, thr):
    """Layer-mean distance of the listed pairs; cand is [Q][C] (pool index or -1), live [P] or None.

    Returns dict(dist [Q][C], best_idx, best_dist, match_idx)."""
    kq, vq, kp, vp = _kv(kq), _kv(vq), _kv(kp), _kv(vp)
    L, Q, T, H, Dh = kq.shape
    P = kp.shape[1]
    cand = np.ascontiguousarray(cand, dtype=np.int32)
    assert cand.ndim == 2 and cand.shape[0] == Q
    C = cand.shape[1]
    if live is not None:
        live = np.ascontiguousarray(live, dtype=np.uint8)
        assert live.shape == (P,)
    D = T * H * Dh
    dist = np.zeros((Q, C), dtype=np.float64)
    best_idx = np.zeros(Q, dtype=np.int32)
    match_idx = np.zeros(Q, dtype=np.int32)
    best = np.zeros(Q, dtype=np.float64)
    rc = _load().rc_oracle_candidate_distances(
        ctypes.c_int(dtype), ctypes.c_int(L), ctypes.c_int(T), ctypes.c_int(H), ctypes.c_int(Dh),
        _p(kq), _p(vq), ctypes.c_int64(Q * D), ctypes.c_int64(Q), _p(kp), _p(vp), ctypes.c_int64(P * D), ctypes.c_int64(P),
        _p(cand), ctypes.c_int64(C), _p(live), ctypes.c_double(thr), _p(dist), _p(best_idx), _p(best), _p(match_idx))
    _check(rc, "candidate_distances")
    return dict(dist=dist, best_idx=best_idx, best_dist=best, match_idx=match_idx)


def pat_threshold(samples, p):
    """Nearest-rank p-th percentile of the finite float32 samples.  Returns (threshold float32, n_finite)."""
    samples = np.ascontiguousarray(samples, dtype=np.float32).ravel()
    thr = np.zeros(1, dtype=np.float32)
    cnt = np.zeros(1, dtype=np.int64)
    rc = _load().rc_oracle_pat_threshold(_p(samples), ctypes.c_int64(samples.size), ctypes.c_double(p), _p(thr), _p(cnt))
    _check(rc, "pat_threshold")
    return thr[0], int(cnt[0])


def apply_threshold(best_idx, best_dist, thr):
    best_idx = np.ascontiguousarray(best_idx, dtype=np.int32).ravel()
    best_dist = np.ascontiguousarray(best_dist, dtype=np.float32).ravel()
    out = np.zeros(best_idx.size, dtype=np.int32)
    rc = _load().rc_oracle_apply_threshold(_p(best_idx), _p(best_dist), ctypes.c_int64(best_idx.size),
                                           ctypes.c_float(thr), _p(out))
    _check(rc, "apply_threshold")
    return out


def pool_admit(kq, vq, q_ksq, q_vsq, kp, vp, p_ksq, p_vsq, live, match_idx):
    """Admit unmatched query blocks into free pool slots.  kp, vp, p_ksq, p_vsq, live are updated IN PLACE
    (uint16 [L][P][T][H][Dh], float64 [L][P] or [L][P][H], uint8 [P]).  Returns (slot_of_query [Q], n_admitted)."""
    kq, vq = _kv(kq), _kv(vq)
    L, Q, T, H, Dh = kq.shape
    P = kp.shape[1]
    for a in (kp, vp):
        assert a.dtype == np.uint16 and a.flags.c_contiguous and a.shape == (L, P, T, H, Dh)
    nh = 1 if q_ksq.ndim == 2 else q_ksq.shape[2]
    q_ksq, q_vsq = np.ascontiguousarray(q_ksq, dtype=np.float64), np.ascontiguousarray(q_vsq, dtype=np.float64)
    for a in (p_ksq, p_vsq):
        assert a.dtype == np.float64 and a.flags.c_contiguous and a.shape[:2] == (L, P)
    assert live.dtype == np.uint8 and live.flags.c_contiguous and live.shape == (P,)
    match_idx = np.ascontiguousarray(match_idx, dtype=np.int32)
    assert match_idx.shape == (Q,)
    slot = np.zeros(Q, dtype=np.int32)
    n = np.zeros(1, dtype=np.int32)
    D = T * H * Dh
    rc = _load().rc_oracle_pool_admit(
        ctypes.c_int(L), ctypes.c_int64(D), ctypes.c_int(nh), _p(kq), _p(vq), ctypes.c_int64(Q * D), ctypes.c_int64(Q),
        _p(q_ksq), _p(q_vsq), _p(kp), _p(vp), ctypes.c_int64(P * D), ctypes.c_int64(P), _p(p_ksq), _p(p_vsq), _p(live),
        _p(match_idx), _p(slot), _p(n))
    _check(rc, "pool_admit")
    return slot, int(n[0])


def pool_touch(slots, value, array):
    """array[slots[i]] = value for the listed slots inside the array (IN PLACE, int32)."""
    slots = np.ascontiguousarray(slots, dtype=np.int32)
    assert array.dtype == np.int32 and array.flags.c_contiguous and array.ndim == 1
    _check(_load().rc_oracle_pool_touch(_p(slots), ctypes.c_int64(slots.size), ctypes.c_int32(int(value)), _p(array),
                                        ctypes.c_int64(array.size)), "pool_touch")
    return array


def refcount_release(ids, refcount):
    """refcount[ids[i]] -= 1 for every listed id inside the array, with multiplicity (IN PLACE, int32)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    assert refcount.dtype == np.int32 and refcount.flags.c_contiguous and refcount.ndim == 1
    _check(_load().rc_oracle_refcount_release(_p(ids), ctypes.c_int64(ids.size), _p(refcount),
                                              ctypes.c_int64(refcount.size)), "refcount_release")
    return refcount


def pool_evict(live, refcount, last_used, match_idx, extra_wanted=0):
    """Make room for the unmatched queries (+ extra_wanted): unreferenced live slots leave in LRU order.
    live (uint8 [P]) is updated IN PLACE; refcount may be None.  Returns (n_free, n_evicted)."""
    assert live.dtype == np.uint8 and live.flags.c_contiguous and live.ndim == 1
    P = live.size
    if refcount is not None:
        refcount = np.ascontiguousarray(refcount, dtype=np.int32)
        assert refcount.shape == (P,)
    last_used = np.ascontiguousarray(last_used, dtype=np.int32)
    assert last_used.shape == (P,)
    match_idx = np.ascontiguousarray(match_idx, dtype=np.int32)
    nf, ne = np.zeros(1, dtype=np.int32), np.zeros(1, dtype=np.int32)
    _check(_load().rc_oracle_pool_evict(ctypes.c_int64(P), _p(live), _p(refcount), _p(last_used), _p(match_idx),
                                        ctypes.c_int64(match_idx.size), ctypes.c_int64(int(extra_wanted)), _p(nf), _p(ne)),
           "pool_evict")
    return int(nf[0]), int(ne[0])


def remap(tables, query_ids, pool_ids, match_idx, P, NB, refcount):
    """Block-table remap.  Returns dict(tables, refcount, freed, n_remapped); inputs are not modified."""
    tables = np.ascontiguousarray(tables, dtype=np.int32)
    assert tables.ndim == 3
    L, R, E = tables.shape
    query_ids = np.ascontiguousarray(query_ids, dtype=np.int32)
    Q = query_ids.size
    match_idx = np.ascontiguousarray(match_idx, dtype=np.int32)
    assert match_idx.shape == (L, Q)
    if pool_ids is not None:
        pool_ids = np.ascontiguousarray(pool_ids, dtype=np.int32)
        assert pool_ids.size == P
    refcount = np.ascontiguousarray(refcount, dtype=np.int32)
    assert refcount.shape == (L, NB)
    tout = np.empty_like(tables)
    rout = np.empty_like(refcount)
    freed = np.zeros((L, Q), dtype=np.uint8)
    nrem = np.zeros((L,), dtype=np.int32)
    rc = _load().rc_oracle_remap(
        ctypes.c_int(L), _p(tables), _p(tout), ctypes.c_int64(R), ctypes.c_int64(E),
        _p(query_ids), _p(pool_ids), _p(match_idx), ctypes.c_int64(Q), ctypes.c_int64(P), ctypes.c_int64(NB),
        _p(refcount), _p(rout), _p(freed), _p(nrem))
    _check(rc, "remap")
    return dict(tables=tout, refcount=rout, freed=freed, n_remapped=nrem)
