"""The C-ABI library loads, exports what include/rc.h declares, and validates arguments on the host.

No kernel is launched here: every call either has nothing to do or fails validation first.
"""
import ctypes
import os
import re

import pytest

from paper_2507_21433_amd import binding as rc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(rc.LIB_PATH):
        from paper_2507_21433_amd import build
        build.build()
    return rc.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "rc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rc_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(rc.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_error_string(lib):
    assert lib.rc_version() >= 100
    assert isinstance(lib.rc_last_error(), bytes)


def desc(L=2, T=16, H=8, Dh=128, dtype=0, stride=None, n=4):
    return rc.KvDesc(L, T, H, Dh, dtype, n * T * H * Dh if stride is None else stride)


FAKE = ctypes.c_void_p(0x1000)      # never dereferenced: validation fails before any launch
ODD = ctypes.c_void_p(0x1004)


def test_norms_validation(lib):
    d = desc()
    assert lib.rc_block_norms(ctypes.byref(d), 0, None, None, 0, None, None, None) == 0     # nothing to do
    assert lib.rc_block_norms(None, 0, FAKE, FAKE, 4, FAKE, FAKE, None) == 1
    assert lib.rc_block_norms(ctypes.byref(d), 0, None, FAKE, 4, FAKE, FAKE, None) == 1
    assert b"NULL" in lib.rc_last_error()
    assert lib.rc_block_norms(ctypes.byref(d), 0, ODD, FAKE, 4, FAKE, FAKE, None) == 1
    assert lib.rc_block_norms(ctypes.byref(d), 0, FAKE, FAKE, -1, FAKE, FAKE, None) == 1
    assert lib.rc_block_norms(ctypes.byref(d), 5, FAKE, FAKE, 4, FAKE, FAKE, None) == 2
    for bad in (desc(Dh=64), desc(T=8), desc(H=17), desc(dtype=3)):
        assert lib.rc_block_norms(ctypes.byref(bad), 0, FAKE, FAKE, 4, FAKE, FAKE, None) == 2
    small = desc(stride=100)
    assert lib.rc_block_norms(ctypes.byref(small), 0, FAKE, FAKE, 4, FAKE, FAKE, None) == 1
    assert lib.rc_block_norms(ctypes.byref(d), 0, FAKE, FAKE, 4, FAKE, FAKE, None) != 99  # (valid call not made)


def test_match_validation(lib):
    q, p = desc(n=4), desc(n=64)
    args = lambda **kw: [kw.get("qd", ctypes.byref(q)), kw.get("pd", ctypes.byref(p)), kw.get("mode", 0),
                         kw.get("kq", FAKE), FAKE, kw.get("Q", 4), FAKE, FAKE, FAKE, FAKE, kw.get("P", 64), FAKE, FAKE,
                         None, kw.get("tau", 0.9), FAKE, FAKE, FAKE, None, kw.get("ws", FAKE), kw.get("wsb", 1 << 26),
                         None]
    # whole tiles: one 16-byte partial per (layer, pool tile, query), then the tile schedule: 520 words of 128 bytes and one claim word per tile slot and workgroup
    # (400 tiles rounded up to whole rounds of 256)
    many = desc(L=200, n=4)
    assert lib.rc_match_workspace_size(ctypes.byref(many), 0, 4, 257) == 200 * 2 * 4 * 16 + (520 * 32 + 512 + 512) * 4
    assert lib.rc_match_workspace_size(ctypes.byref(many), 1, 4, 257) == 200 * 2 * 4 * 16 + (520 * 32 + 512 + 512) * 4
    # per-head mode with few tiles: one share of 256 KB per head and tile, then the partials of the pool chunks
    assert lib.rc_match_workspace_size(ctypes.byref(q), 1, 4, 64) == 2 * 8 * 65536 * 4 + 2 * 2 * 4 * 16
    assert lib.rc_match_workspace_size(ctypes.byref(q), 1, 4, 257) == 2 * 8 * 2 * 65536 * 4 + 2 * 9 * 4 * 16
    # block mode with few tiles: 2 tiles x 64 shares of 256 KB, then 2 pool chunks of partials per layer
    assert lib.rc_match_workspace_size(ctypes.byref(q), 0, 4, 64) == 2 * 64 * 65536 * 4 + 2 * 2 * 4 * 16
    assert lib.rc_match_workspace_size(ctypes.byref(q), 9, 4, 64) == 0
    assert lib.rc_match_blocks(*args(Q=0)) == 0                      # nothing to do
    assert lib.rc_match_blocks(*args(wsb=8)) == 3
    assert b"workspace" in lib.rc_last_error()
    assert lib.rc_match_blocks(*args(ws=None)) == 3
    assert lib.rc_match_blocks(*args(kq=None)) == 1
    assert lib.rc_match_blocks(*args(kq=ODD)) == 1
    assert lib.rc_match_blocks(*args(tau=float("nan"))) == 1
    assert lib.rc_match_blocks(*args(mode=2)) == 2
    other = desc(n=64, T=32)
    assert lib.rc_match_blocks(*args(pd=ctypes.byref(other))) == 1
    assert lib.rc_match_blocks(*args(Q=-1)) == 1


def test_remap_validation(lib):
    args = lambda **kw: [kw.get("L", 2), FAKE, FAKE, kw.get("R", 4), kw.get("E", 8), FAKE, kw.get("pids", None), FAKE,
                         kw.get("Q", 4), kw.get("P", 16), kw.get("NB", 20), kw.get("rin", FAKE), FAKE, FAKE, FAKE,
                         kw.get("ws", FAKE), kw.get("wsb", 1 << 20), None]
    need = lib.rc_remap_workspace_size(2, 4, 8, 4, 20)
    assert need == 20 * 4                           # the reverse index; one workgroup per layer keeps its counts in LDS
    # two layers of 800 000 entries are cut into 128 chunks each (256 workgroups): one histogram of Q counts per chunk and layer
    assert lib.rc_remap_workspace_size(2, 8, 100000, 4, 20) == 20 * 4 + 2 * 128 * 4 * 4
    assert lib.rc_remap_block_table(*args(L=0)) == 0
    assert lib.rc_remap_block_table(*args(wsb=need - 1)) == 3
    assert lib.rc_remap_block_table(*args(Q=8193)) == 2
    assert lib.rc_remap_block_table(*args(P=21)) == 1                 # identity pool ids need P <= NB
    assert lib.rc_remap_block_table(*args(rin=None)) == 1
    assert lib.rc_remap_block_table(*args(R=-1)) == 1


def test_candidates_validation(lib):
    q, p = desc(n=4), desc(n=64)
    args = lambda **kw: [kw.get("qd", ctypes.byref(q)), ctypes.byref(p), kw.get("mode", 0), kw.get("kq", FAKE), FAKE,
                         kw.get("Q", 4), FAKE, FAKE, FAKE, FAKE, 64, FAKE, FAKE, None, kw.get("cand", FAKE),
                         kw.get("C", 3), kw.get("tau", 0.9), kw.get("scores", FAKE), FAKE, FAKE, FAKE, None]
    assert lib.rc_score_candidates(*args(Q=0)) == 0
    assert lib.rc_score_candidates(*args(C=-1)) == 1
    assert lib.rc_score_candidates(*args(cand=None)) == 1
    assert lib.rc_score_candidates(*args(scores=None)) == 1
    assert lib.rc_score_candidates(*args(kq=ODD)) == 1
    assert lib.rc_score_candidates(*args(tau=float("nan"))) == 1
    assert lib.rc_score_candidates(*args(mode=7)) == 2
    h3 = desc(n=4, H=3)
    assert lib.rc_score_candidates(*args(qd=ctypes.byref(h3), mode=1)) == 1           # query and pool descriptors differ
    # layer-mean distance of listed pairs
    dargs = lambda **kw: [kw.get("qd", ctypes.byref(q)), ctypes.byref(p), kw.get("kq", FAKE), FAKE, kw.get("Q", 4), FAKE, FAKE,
                          64, None, kw.get("cand", FAKE), kw.get("C", 3), kw.get("thr", 0.5), FAKE, FAKE, FAKE, FAKE,
                          kw.get("ws", FAKE), kw.get("wsb", 1 << 20), None]
    assert lib.rc_candidate_distances_workspace_size(ctypes.byref(q), 4, 3) >= 4 * 3 * 4
    zero_layers = desc(L=0, n=4)
    assert lib.rc_candidate_distances_workspace_size(ctypes.byref(zero_layers), 4, 3) == 0
    assert lib.rc_candidate_distances(*dargs(Q=0)) == 0
    assert lib.rc_candidate_distances(*dargs(wsb=4)) == 3
    assert lib.rc_candidate_distances(*dargs(thr=float("nan"))) == 1
    assert lib.rc_candidate_distances(*dargs(cand=None)) == 1
    assert lib.rc_candidate_distances(*dargs(kq=None)) == 1


def test_layer_mean_pat_and_pool_validation(lib):
    q, p = desc(n=4), desc(n=64)
    largs = lambda **kw: [kw.get("qd", ctypes.byref(q)), kw.get("pd", ctypes.byref(p)), kw.get("kq", FAKE), FAKE, kw.get("Q", 4),
                          FAKE, FAKE, FAKE, FAKE, 64, FAKE, FAKE, None, kw.get("thr", 0.5), FAKE, FAKE, FAKE, None,
                          kw.get("ws", FAKE), kw.get("wsb", 1 << 30), None]
    assert lib.rc_layer_mean_workspace_size(ctypes.byref(q), 4, 64) >= 65536 * 4
    assert lib.rc_match_blocks_layer_mean(*largs(Q=0)) == 0
    assert lib.rc_match_blocks_layer_mean(*largs(wsb=1024)) == 3
    assert lib.rc_match_blocks_layer_mean(*largs(thr=float("nan"))) == 1
    assert lib.rc_match_blocks_layer_mean(*largs(kq=None)) == 1
    z = desc(L=0, n=4)
    zp = desc(L=0, n=64)
    assert lib.rc_match_blocks_layer_mean(*largs(qd=ctypes.byref(z), pd=ctypes.byref(zp))) == 1   # a mean over no layers
    assert b"layers" in lib.rc_last_error()
    # percentile
    assert lib.rc_pat_workspace_size() >= 4 * 256 * 4
    pargs = lambda **kw: [kw.get("s", FAKE), kw.get("n", 10), kw.get("p", 80.0), kw.get("thr", FAKE), None,
                          kw.get("ws", FAKE), kw.get("wsb", 1 << 16), None]
    assert lib.rc_pat_threshold(*pargs(p=100.5)) == 1
    assert lib.rc_pat_threshold(*pargs(p=-1.0)) == 1
    assert lib.rc_pat_threshold(*pargs(p=float("nan"))) == 1
    assert lib.rc_pat_threshold(*pargs(n=-1)) == 1
    assert lib.rc_pat_threshold(*pargs(n=1 << 31)) == 1
    assert lib.rc_pat_threshold(*pargs(thr=None)) == 1
    assert lib.rc_pat_threshold(*pargs(s=None)) == 1
    assert lib.rc_pat_threshold(*pargs(wsb=16)) == 3
    assert lib.rc_apply_threshold(FAKE, FAKE, 0, FAKE, FAKE, None) == 0
    assert lib.rc_apply_threshold(FAKE, FAKE, -1, FAKE, FAKE, None) == 1
    assert lib.rc_apply_threshold(FAKE, FAKE, 5, None, FAKE, None) == 1
    # admission
    aargs = lambda **kw: [ctypes.byref(q), ctypes.byref(p), kw.get("mode", 0), kw.get("kq", FAKE), FAKE, 4, FAKE, FAKE, FAKE, FAKE,
                          64, FAKE, FAKE, kw.get("live", FAKE), kw.get("m", FAKE), FAKE, kw.get("n", FAKE),
                          kw.get("ws", FAKE), kw.get("wsb", 1 << 20), None]
    assert lib.rc_pool_admit_workspace_size(4, 64) > 0 and lib.rc_pool_admit_workspace_size(-1, 64) == 0
    assert lib.rc_pool_admit(*aargs(n=None)) == 1
    assert lib.rc_pool_admit(*aargs(m=None)) == 1
    assert lib.rc_pool_admit(*aargs(live=None)) == 1
    assert lib.rc_pool_admit(*aargs(kq=ODD)) == 1
    assert lib.rc_pool_admit(*aargs(mode=3)) == 2
    assert lib.rc_pool_admit(*aargs(wsb=8)) == 3


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(rc, "_lib", None)
    monkeypatch.setattr(rc, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        rc.lib()
