"""rc_remap_block_table_static (the entry point that allocates nothing) against rc_remap_block_table.

Two calls in a row on the library's built-in scratch buffer, the second on a smaller problem, each
compared bit by bit with the entry point that takes a caller-owned workspace; then a problem that
exceeds the buffer, which must be refused before anything is launched.
"""
import ctypes

import numpy as np
import pytest
import torch

from paper_2507_21433_amd import binding as rc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def problem(seed, L, R, E, Q, P, shared_targets=False):
    g = np.random.RandomState(seed)
    NB = P + Q + 37
    ids = g.permutation(NB).astype(np.int32)
    query_ids, pool_ids = ids[:Q].copy(), ids[Q:Q + P].copy()
    tables = g.randint(0, NB, size=(L, R, E)).astype(np.int32)
    hit = g.rand(L, R, E) < 0.3
    tables[hit] = query_ids[g.randint(0, Q, size=int(hit.sum()))]
    tables[g.rand(L, R, E) < 0.05] = -1
    match = g.randint(0, 8 if shared_targets else P, size=(L, Q)).astype(np.int32)
    match[g.rand(L, Q) < 0.4] = -1
    refcount = np.stack([np.bincount(t[t >= 0].ravel(), minlength=NB) for t in tables]).astype(np.int32)
    refcount += g.randint(0, 2, size=refcount.shape).astype(np.int32)   # some references held outside the tables
    t = lambda a: torch.as_tensor(a, device=DEV)
    return dict(tables=t(tables), query_ids=t(query_ids), pool_ids=t(pool_ids), match=t(match), refcount=t(refcount),
                P=P, NB=NB, L=L, Q=Q)


def outputs(pr):
    return dict(tables=torch.full_like(pr["tables"], -7), refcount=torch.full_like(pr["refcount"], -7),
                freed=torch.full((pr["L"], pr["Q"]), 9, dtype=torch.uint8, device=DEV),
                n_remapped=torch.full((pr["L"],), -7, dtype=torch.int32, device=DEV))


def run_both(pr):
    want = rc.rc_remap_block_table(pr["tables"], pr["query_ids"], pr["pool_ids"], pr["match"], pr["P"], pr["NB"],
                                   pr["refcount"], out=outputs(pr))
    got = rc.rc_remap_block_table_static(pr["tables"], pr["query_ids"], pr["pool_ids"], pr["match"], pr["P"], pr["NB"],
                                         pr["refcount"], out=outputs(pr))
    torch.cuda.synchronize()
    for k in ("tables", "refcount", "freed", "n_remapped"):
        assert torch.equal(got[k], want[k]), k
    assert int(want["n_remapped"].sum()) > 0


def test_static_scratch_matches_workspace_entry_point_twice_in_a_row():
    print("[gpu-case] rc_remap_block_table_static: 6 layers x 40 x 700 entries, Q=900, P=5000", flush=True)
    big = problem(11, L=6, R=40, E=700, Q=900, P=5000)
    run_both(big)
    print("[gpu-case] rc_remap_block_table_static: second call, smaller: 2 layers x 3 x 50 entries, Q=70, P=90", flush=True)
    small = problem(12, L=2, R=3, E=50, Q=70, P=90, shared_targets=True)
    run_both(small)
    # and the larger one once more over whatever the small call left in the buffer
    run_both(big)


def test_static_scratch_refuses_what_does_not_fit():
    lib = rc.lib()
    cap = lib.rc_remap_static_scratch_size()
    assert cap == 4 << 20
    L, R, E, Q, NB = 64, 64, 776, 1024, 2_000_000
    assert lib.rc_remap_workspace_size(L, R, E, Q, NB) > cap
    fake = ctypes.c_void_p(0x1000)        # never dereferenced: refused on the host
    code = lib.rc_remap_block_table_static(L, fake, fake, R, E, fake, None, fake, Q, 1000, NB, fake, fake, fake, fake, None)
    assert code == 3 and b"built-in buffer" in lib.rc_last_error()
