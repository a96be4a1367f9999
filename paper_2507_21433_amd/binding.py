"""Thin ctypes binding of the C-ABI HIP library (``include/rc.h``).

Argument marshalling only: every step of the search runs in the HIP kernels.
PyTorch supplies device memory and the current stream.  There is no CPU
fallback: if ``librc.so`` has not been built the first call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librc.so")

RC_OK = 0
RC_F16, RC_BF16 = 0, 1
RC_SCORE_BLOCK, RC_SCORE_PER_HEAD_ALL = 0, 1

EXPORTS = ("rc_block_norms", "rc_match_workspace_size", "rc_match_blocks", "rc_remap_workspace_size",
           "rc_remap_block_table", "rc_remap_static_scratch_size", "rc_remap_block_table_static", "rc_score_candidates", "rc_layer_mean_workspace_size", "rc_match_blocks_layer_mean",
           "rc_pat_workspace_size", "rc_pat_threshold", "rc_apply_threshold", "rc_pool_admit_workspace_size", "rc_pool_admit",
           "rc_candidate_distances_workspace_size", "rc_candidate_distances", "rc_pool_touch", "rc_refcount_release", "rc_pool_evict",
           "rc_last_error", "rc_version")


class RcError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"rc status {code}: {text}")
        self.code = code


class KvDesc(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("block_tokens", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("layer_stride", ctypes.c_int64)]


_lib = None


def lib():
    """Load ``librc.so`` (built by ``paper_2507_21433_amd.build``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2507_21433_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
        dp = ctypes.POINTER(KvDesc)
        L.rc_block_norms.argtypes = [dp, i32, vp, vp, i64, vp, vp, vp]
        L.rc_block_norms.restype = i32
        L.rc_match_workspace_size.argtypes = [dp, i32, i64, i64]
        L.rc_match_workspace_size.restype = sz
        L.rc_match_blocks.argtypes = [dp, dp, i32, vp, vp, i64, vp, vp, vp, vp, i64, vp, vp, vp, f32,
                                      vp, vp, vp, vp, vp, sz, vp]
        L.rc_match_blocks.restype = i32
        L.rc_remap_workspace_size.argtypes = [i32, i64, i64, i64, i64]
        L.rc_remap_workspace_size.restype = sz
        L.rc_remap_block_table.argtypes = [i32, vp, vp, i64, i64, vp, vp, vp, i64, i64, i64, vp, vp, vp, vp,
                                           vp, sz, vp]
        L.rc_remap_block_table.restype = i32
        L.rc_remap_static_scratch_size.argtypes = []
        L.rc_remap_static_scratch_size.restype = sz
        L.rc_remap_block_table_static.argtypes = [i32, vp, vp, i64, i64, vp, vp, vp, i64, i64, i64, vp, vp, vp, vp, vp]
        L.rc_remap_block_table_static.restype = i32
        L.rc_score_candidates.argtypes = [dp, dp, i32, vp, vp, i64, vp, vp, vp, vp, i64, vp, vp, vp, vp, i64, f32,
                                          vp, vp, vp, vp, vp]
        L.rc_score_candidates.restype = i32
        L.rc_layer_mean_workspace_size.argtypes = [dp, i64, i64]
        L.rc_layer_mean_workspace_size.restype = sz
        L.rc_match_blocks_layer_mean.argtypes = [dp, dp, vp, vp, i64, vp, vp, vp, vp, i64, vp, vp, vp, f32,
                                                 vp, vp, vp, vp, vp, sz, vp]
        L.rc_match_blocks_layer_mean.restype = i32
        L.rc_pat_workspace_size.argtypes = []
        L.rc_pat_workspace_size.restype = sz
        L.rc_pat_threshold.argtypes = [vp, i64, ctypes.c_double, vp, vp, vp, sz, vp]
        L.rc_pat_threshold.restype = i32
        L.rc_apply_threshold.argtypes = [vp, vp, i64, vp, vp, vp]
        L.rc_apply_threshold.restype = i32
        L.rc_pool_admit_workspace_size.argtypes = [i64, i64]
        L.rc_pool_admit_workspace_size.restype = sz
        L.rc_pool_admit.argtypes = [dp, dp, i32, vp, vp, i64, vp, vp, vp, vp, i64, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.rc_pool_admit.restype = i32
        L.rc_candidate_distances_workspace_size.argtypes = [dp, i64, i64]
        L.rc_candidate_distances_workspace_size.restype = sz
        L.rc_candidate_distances.argtypes = [dp, dp, vp, vp, i64, vp, vp, i64, vp, vp, i64, f32, vp, vp, vp, vp, vp, sz, vp]
        L.rc_candidate_distances.restype = i32
        L.rc_pool_touch.argtypes = [vp, i64, i32, vp, i64, vp]
        L.rc_pool_touch.restype = i32
        L.rc_refcount_release.argtypes = [vp, i64, vp, i64, vp]
        L.rc_refcount_release.restype = i32
        L.rc_pool_evict.argtypes = [i64, vp, vp, vp, vp, i64, i64, vp, vp, vp]
        L.rc_pool_evict.restype = i32
        L.rc_last_error.restype = ctypes.c_char_p
        L.rc_version.restype = i32
        _lib = L
    return _lib


def _check(code):
    if code != RC_OK:
        raise RcError(code, lib().rc_last_error().decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t):
    if t.dtype == torch.float16:
        return RC_F16
    if t.dtype == torch.bfloat16:
        return RC_BF16
    raise TypeError(f"KV dtype {t.dtype} (fp16 or bf16 only)")


def kv_desc(t):
    """Descriptor of a KV tensor shaped [L][n][T][H][Dh] whose inner four dims are contiguous."""
    assert t.dim() == 5, "KV tensors are [L][n][T][H][Dh]"
    L, n, T, H, Dh = t.shape
    assert t[0].is_contiguous(), "blocks of a layer must be contiguous"
    stride = t.stride(0) if L > 1 else n * T * H * Dh
    return KvDesc(L, T, H, Dh, _dtype_code(t), stride)


def _dev(*ts):
    for t in ts:
        assert t is None or t.is_cuda, "device tensors only"


def rc_block_norms(k, v, mode=RC_SCORE_BLOCK, k_sqnorm=None, v_sqnorm=None):
    """Squared norms of every block: returns (k_sqnorm, v_sqnorm), fp32 [L][n] or [L][n][H]."""
    _dev(k, v)
    d = kv_desc(k)
    assert v.shape == k.shape and v.dtype == k.dtype and kv_desc(v).layer_stride == d.layer_stride
    L, n, H = k.shape[0], k.shape[1], k.shape[3]
    shape = (L, n) if mode == RC_SCORE_BLOCK else (L, n, H)
    if k_sqnorm is None:
        k_sqnorm = torch.empty(shape, dtype=torch.float32, device=k.device)
    if v_sqnorm is None:
        v_sqnorm = torch.empty(shape, dtype=torch.float32, device=k.device)
    assert k_sqnorm.shape == shape and v_sqnorm.shape == shape and k_sqnorm.is_contiguous() and v_sqnorm.is_contiguous()
    _check(lib().rc_block_norms(ctypes.byref(d), mode, _ptr(k), _ptr(v), n, _ptr(k_sqnorm), _ptr(v_sqnorm), _stream()))
    return k_sqnorm, v_sqnorm


def rc_match_workspace_size(kq, mode, Q, P):
    d = kv_desc(kq)
    return lib().rc_match_workspace_size(ctypes.byref(d), mode, Q, P)


def rc_match_blocks(kq, vq, q_ksq, q_vsq, kp, vp, p_ksq, p_vsq, pool_live, tau, mode=RC_SCORE_BLOCK,
                    want_second=True, workspace=None, out=None):
    """Best live pool block per query.  Returns dict(best_idx, best_score, match_idx, second_score)."""
    _dev(kq, vq, kp, vp, q_ksq, q_vsq, p_ksq, p_vsq, pool_live)
    qd, pd = kv_desc(kq), kv_desc(kp)
    assert kv_desc(vq).layer_stride == qd.layer_stride and kv_desc(vp).layer_stride == pd.layer_stride
    L, Q, P = kq.shape[0], kq.shape[1], kp.shape[1]
    for t in (q_ksq, q_vsq, p_ksq, p_vsq):
        assert t.dtype == torch.float32 and t.is_contiguous()
    if pool_live is not None:
        assert pool_live.dtype == torch.uint8 and pool_live.shape == (L, P) and pool_live.is_contiguous()
    need = lib().rc_match_workspace_size(ctypes.byref(qd), mode, Q, P)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=kq.device)
    if out is None:
        out = dict(best_idx=torch.empty((L, Q), dtype=torch.int32, device=kq.device),
                   best_score=torch.empty((L, Q), dtype=torch.float32, device=kq.device),
                   match_idx=torch.empty((L, Q), dtype=torch.int32, device=kq.device),
                   second_score=torch.empty((L, Q), dtype=torch.float32, device=kq.device) if want_second else None)
    _check(lib().rc_match_blocks(ctypes.byref(qd), ctypes.byref(pd), mode, _ptr(kq), _ptr(vq), Q, _ptr(q_ksq),
                                 _ptr(q_vsq), _ptr(kp), _ptr(vp), P, _ptr(p_ksq), _ptr(p_vsq), _ptr(pool_live),
                                 float(tau), _ptr(out["best_idx"]), _ptr(out["best_score"]), _ptr(out["match_idx"]),
                                 _ptr(out.get("second_score")), _ptr(workspace), workspace.numel(), _stream()))
    return out


def rc_remap_workspace_size(L, R, E, Q, NB):
    return lib().rc_remap_workspace_size(L, R, E, Q, NB)


def rc_remap_block_table(tables, query_ids, pool_ids, match_idx, P, NB, refcount, in_place=False, workspace=None,
                         out=None):
    """Redirect table entries of matched query blocks.  Returns dict(tables, refcount, freed, n_remapped)."""
    _dev(tables, query_ids, pool_ids, match_idx, refcount)
    assert tables.dtype == torch.int32 and tables.dim() == 3 and tables.is_contiguous()
    L, R, E = tables.shape
    Q = query_ids.numel()
    assert query_ids.dtype == torch.int32 and match_idx.dtype == torch.int32 and match_idx.shape == (L, Q)
    assert match_idx.is_contiguous() and refcount.dtype == torch.int32 and refcount.shape == (L, NB)
    assert refcount.is_contiguous()
    if pool_ids is not None:
        assert pool_ids.dtype == torch.int32 and pool_ids.numel() == P
    if out is not None:
        t_out, r_out, freed, n_remapped = out["tables"], out["refcount"], out["freed"], out["n_remapped"]
    else:
        t_out = tables if in_place else torch.empty_like(tables)
        r_out = refcount if in_place else torch.empty_like(refcount)
        freed = torch.empty((L, Q), dtype=torch.uint8, device=tables.device)
        n_remapped = torch.empty((L,), dtype=torch.int32, device=tables.device)
    need = lib().rc_remap_workspace_size(L, R, E, Q, NB)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=tables.device)
    _check(lib().rc_remap_block_table(L, _ptr(tables), _ptr(t_out), R, E, _ptr(query_ids), _ptr(pool_ids),
                                      _ptr(match_idx), Q, P, NB, _ptr(refcount), _ptr(r_out), _ptr(freed),
                                      _ptr(n_remapped), _ptr(workspace), workspace.numel(), _stream()))
    return dict(tables=t_out, refcount=r_out, freed=freed, n_remapped=n_remapped)


def rc_remap_block_table_static(tables, query_ids, pool_ids, match_idx, P, NB, refcount, out):
    """rc_remap_block_table on the library's built-in scratch buffer: no workspace, and every output is the caller's (`out`)."""
    _dev(tables, query_ids, pool_ids, match_idx, refcount, out["tables"], out["refcount"], out["freed"], out["n_remapped"])
    assert tables.dtype == torch.int32 and tables.dim() == 3 and tables.is_contiguous()
    L, R, E = tables.shape
    Q = query_ids.numel()
    assert query_ids.dtype == torch.int32 and match_idx.dtype == torch.int32 and match_idx.shape == (L, Q)
    assert match_idx.is_contiguous() and refcount.dtype == torch.int32 and refcount.shape == (L, NB)
    assert refcount.is_contiguous()
    if pool_ids is not None:
        assert pool_ids.dtype == torch.int32 and pool_ids.numel() == P
    assert out["tables"].shape == tables.shape and out["refcount"].shape == refcount.shape
    assert out["freed"].shape == (L, Q) and out["freed"].dtype == torch.uint8 and out["n_remapped"].shape == (L,)
    _check(lib().rc_remap_block_table_static(L, _ptr(tables), _ptr(out["tables"]), R, E, _ptr(query_ids), _ptr(pool_ids),
                                             _ptr(match_idx), Q, P, NB, _ptr(refcount), _ptr(out["refcount"]),
                                             _ptr(out["freed"]), _ptr(out["n_remapped"]), _stream()))
    return out


def rc_score_candidates(kq, vq, q_ksq, q_vsq, kp, vp, p_ksq, p_vsq, pool_live, cand, tau, mode=RC_SCORE_BLOCK, out=None):
    """Scores of the listed candidates [L][Q][C].  Returns dict(scores, best_idx, best_score, match_idx)."""
    _dev(kq, vq, kp, vp, q_ksq, q_vsq, p_ksq, p_vsq, pool_live, cand)
    qd, pd = kv_desc(kq), kv_desc(kp)
    L, Q, P = kq.shape[0], kq.shape[1], kp.shape[1]
    assert cand.dtype == torch.int32 and cand.dim() == 3 and cand.shape[:2] == (L, Q) and cand.is_contiguous()
    C = cand.shape[2]
    if pool_live is not None:
        assert pool_live.dtype == torch.uint8 and pool_live.shape == (L, P) and pool_live.is_contiguous()
    if out is None:
        out = dict(scores=torch.empty((L, Q, C), dtype=torch.float32, device=kq.device),
                   best_idx=torch.empty((L, Q), dtype=torch.int32, device=kq.device),
                   best_score=torch.empty((L, Q), dtype=torch.float32, device=kq.device),
                   match_idx=torch.empty((L, Q), dtype=torch.int32, device=kq.device))
    _check(lib().rc_score_candidates(ctypes.byref(qd), ctypes.byref(pd), mode, _ptr(kq), _ptr(vq), Q, _ptr(q_ksq),
                                     _ptr(q_vsq), _ptr(kp), _ptr(vp), P, _ptr(p_ksq), _ptr(p_vsq), _ptr(pool_live),
                                     _ptr(cand), C, float(tau), _ptr(out["scores"]), _ptr(out["best_idx"]),
                                     _ptr(out["best_score"]), _ptr(out["match_idx"]), _stream()))
    return out


def rc_layer_mean_workspace_size(kq, Q, P):
    d = kv_desc(kq)
    return lib().rc_layer_mean_workspace_size(ctypes.byref(d), Q, P)


def rc_match_blocks_layer_mean(kq, vq, q_ksq, q_vsq, kp, vp, p_ksq, p_vsq, pool_live, threshold, want_second=True,
                               workspace=None, out=None):
    """Nearest live pool block per query by the layer-mean distance.  Returns dict(best_idx, best_dist, match_idx, second_dist), [Q]."""
    _dev(kq, vq, kp, vp, q_ksq, q_vsq, p_ksq, p_vsq, pool_live)
    qd, pd = kv_desc(kq), kv_desc(kp)
    assert kv_desc(vq).layer_stride == qd.layer_stride and kv_desc(vp).layer_stride == pd.layer_stride
    L, Q, P = kq.shape[0], kq.shape[1], kp.shape[1]
    for t, n in ((q_ksq, Q), (q_vsq, Q), (p_ksq, P), (p_vsq, P)):
        assert t.dtype == torch.float32 and t.is_contiguous() and t.shape == (L, n)
    if pool_live is not None:
        assert pool_live.dtype == torch.uint8 and pool_live.shape == (P,) and pool_live.is_contiguous()
    need = lib().rc_layer_mean_workspace_size(ctypes.byref(qd), Q, P)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=kq.device)
    if out is None:
        out = dict(best_idx=torch.empty((Q,), dtype=torch.int32, device=kq.device),
                   best_dist=torch.empty((Q,), dtype=torch.float32, device=kq.device),
                   match_idx=torch.empty((Q,), dtype=torch.int32, device=kq.device),
                   second_dist=torch.empty((Q,), dtype=torch.float32, device=kq.device) if want_second else None)
    _check(lib().rc_match_blocks_layer_mean(ctypes.byref(qd), ctypes.byref(pd), _ptr(kq), _ptr(vq), Q, _ptr(q_ksq),
                                            _ptr(q_vsq), _ptr(kp), _ptr(vp), P, _ptr(p_ksq), _ptr(p_vsq),
                                            _ptr(pool_live), float(threshold), _ptr(out["best_idx"]),
                                            _ptr(out["best_dist"]), _ptr(out["match_idx"]), _ptr(out.get("second_dist")),
                                            _ptr(workspace), workspace.numel(), _stream()))
    return out


def rc_pat_threshold(samples, p, workspace=None, out=None):
    """Nearest-rank p-th percentile of the finite samples.  Returns dict(threshold float32 [1], n_finite int64 [1]) on the device."""
    _dev(samples)
    assert samples.dtype == torch.float32 and samples.is_contiguous()
    if workspace is None:
        workspace = torch.empty(lib().rc_pat_workspace_size(), dtype=torch.uint8, device=samples.device)
    if out is None:
        out = dict(threshold=torch.empty(1, dtype=torch.float32, device=samples.device),
                   n_finite=torch.empty(1, dtype=torch.int64, device=samples.device))
    _check(lib().rc_pat_threshold(_ptr(samples), samples.numel(), float(p), _ptr(out["threshold"]), _ptr(out["n_finite"]),
                                  _ptr(workspace), workspace.numel(), _stream()))
    return out


def rc_apply_threshold(best_idx, best_dist, threshold, match_idx=None):
    """match_idx = best_idx where best_dist <= threshold (a device scalar), else -1."""
    _dev(best_idx, best_dist, threshold)
    assert best_idx.dtype == torch.int32 and best_dist.dtype == torch.float32 and threshold.dtype == torch.float32
    assert best_idx.is_contiguous() and best_dist.is_contiguous() and best_idx.shape == best_dist.shape
    assert threshold.numel() == 1
    if match_idx is None:
        match_idx = torch.empty_like(best_idx)
    _check(lib().rc_apply_threshold(_ptr(best_idx), _ptr(best_dist), best_idx.numel(), _ptr(threshold), _ptr(match_idx),
                                    _stream()))
    return match_idx


def rc_pool_admit(kq, vq, q_ksq, q_vsq, kp, vp, p_ksq, p_vsq, pool_live, match_idx, mode=RC_SCORE_BLOCK, workspace=None,
                  out=None):
    """Admit unmatched query blocks into free pool slots; kp, vp, p_ksq, p_vsq, pool_live are updated in place.

    Returns dict(slot_of_query int32 [Q], n_admitted int32 [1])."""
    _dev(kq, vq, kp, vp, q_ksq, q_vsq, p_ksq, p_vsq, pool_live, match_idx)
    qd, pd = kv_desc(kq), kv_desc(kp)
    assert kv_desc(vq).layer_stride == qd.layer_stride and kv_desc(vp).layer_stride == pd.layer_stride
    L, Q, P, H = kq.shape[0], kq.shape[1], kp.shape[1], kq.shape[3]
    qs, ps = ((L, Q), (L, P)) if mode == RC_SCORE_BLOCK else ((L, Q, H), (L, P, H))
    for t, sh in ((q_ksq, qs), (q_vsq, qs), (p_ksq, ps), (p_vsq, ps)):
        assert t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == sh
    assert pool_live.dtype == torch.uint8 and pool_live.shape == (P,) and pool_live.is_contiguous()
    assert match_idx.dtype == torch.int32 and match_idx.shape == (Q,) and match_idx.is_contiguous()
    if workspace is None:
        workspace = torch.empty(max(16, lib().rc_pool_admit_workspace_size(Q, P)), dtype=torch.uint8, device=kq.device)
    if out is None:
        out = dict(slot_of_query=torch.empty((Q,), dtype=torch.int32, device=kq.device),
                   n_admitted=torch.empty((1,), dtype=torch.int32, device=kq.device))
    _check(lib().rc_pool_admit(ctypes.byref(qd), ctypes.byref(pd), mode, _ptr(kq), _ptr(vq), Q, _ptr(q_ksq), _ptr(q_vsq),
                               _ptr(kp), _ptr(vp), P, _ptr(p_ksq), _ptr(p_vsq), _ptr(pool_live), _ptr(match_idx),
                               _ptr(out["slot_of_query"]), _ptr(out["n_admitted"]), _ptr(workspace), workspace.numel(),
                               _stream()))
    return out


def rc_candidate_distances(kq, vq, kp, vp, pool_live, cand, threshold, workspace=None, out=None):
    """Layer-mean distance of the listed pairs, cand [Q][C].  Returns dict(dist [Q][C], best_idx, best_dist, match_idx)."""
    _dev(kq, vq, kp, vp, pool_live, cand)
    qd, pd = kv_desc(kq), kv_desc(kp)
    assert kv_desc(vq).layer_stride == qd.layer_stride and kv_desc(vp).layer_stride == pd.layer_stride
    Q, P = kq.shape[1], kp.shape[1]
    assert cand.dtype == torch.int32 and cand.dim() == 2 and cand.shape[0] == Q and cand.is_contiguous()
    C = cand.shape[1]
    if pool_live is not None:
        assert pool_live.dtype == torch.uint8 and pool_live.shape == (P,) and pool_live.is_contiguous()
    if workspace is None:
        workspace = torch.empty(max(16, lib().rc_candidate_distances_workspace_size(ctypes.byref(qd), Q, C)),
                                dtype=torch.uint8, device=kq.device)
    if out is None:
        out = dict(dist=torch.empty((Q, C), dtype=torch.float32, device=kq.device),
                   best_idx=torch.empty((Q,), dtype=torch.int32, device=kq.device),
                   best_dist=torch.empty((Q,), dtype=torch.float32, device=kq.device),
                   match_idx=torch.empty((Q,), dtype=torch.int32, device=kq.device))
    _check(lib().rc_candidate_distances(ctypes.byref(qd), ctypes.byref(pd), _ptr(kq), _ptr(vq), Q, _ptr(kp), _ptr(vp), P,
                                        _ptr(pool_live), _ptr(cand), C, float(threshold), _ptr(out["dist"]),
                                        _ptr(out["best_idx"]), _ptr(out["best_dist"]), _ptr(out["match_idx"]),
                                        _ptr(workspace), workspace.numel(), _stream()))
    return out


def rc_pool_touch(slots, value, array):
    """array[slots[i]] = value for the listed slots inside the array (in place; int32 device tensors)."""
    _dev(slots, array)
    assert slots.dtype == torch.int32 and array.dtype == torch.int32 and slots.is_contiguous() and array.is_contiguous()
    _check(lib().rc_pool_touch(_ptr(slots), slots.numel(), int(value), _ptr(array), array.numel(), _stream()))
    return array


def rc_refcount_release(ids, refcount):
    """refcount[ids[i]] -= 1 for every listed id inside the array, with multiplicity (in place)."""
    _dev(ids, refcount)
    assert ids.dtype == torch.int32 and refcount.dtype == torch.int32 and ids.is_contiguous() and refcount.is_contiguous()
    _check(lib().rc_refcount_release(_ptr(ids), ids.numel(), _ptr(refcount), refcount.numel(), _stream()))
    return refcount


def rc_pool_evict(pool_live, refcount, last_used, match_idx, extra_wanted=0, out=None):
    """Make room for the step's unmatched queries: unreferenced live slots leave in LRU order (pool_live in place).

    Returns dict(n_free int32 [1], n_evicted int32 [1]) on the device."""
    _dev(pool_live, refcount, last_used, match_idx)
    P = pool_live.numel()
    assert pool_live.dtype == torch.uint8 and pool_live.is_contiguous()
    assert last_used.dtype == torch.int32 and last_used.is_contiguous() and last_used.numel() == P
    if refcount is not None:
        assert refcount.dtype == torch.int32 and refcount.is_contiguous() and refcount.numel() == P
    assert match_idx.dtype == torch.int32 and match_idx.is_contiguous()
    if out is None:
        out = dict(n_free=torch.empty(1, dtype=torch.int32, device=pool_live.device),
                   n_evicted=torch.empty(1, dtype=torch.int32, device=pool_live.device))
    _check(lib().rc_pool_evict(P, _ptr(pool_live), _ptr(refcount), _ptr(last_used), _ptr(match_idx), match_idx.numel(),
                               int(extra_wanted), _ptr(out["n_free"]), _ptr(out["n_evicted"]), _stream()))
    return out
