"""The library allocates nothing, synchronises nothing and clears memory with kernels only, so a whole step can be
recorded into a HIP graph.  The graph is replayed several times with eager work and synchronisations in between and
every replay is compared with the eager result, bit by bit.  Needs a real MI355X."""
import sys

import pytest
import torch

from paper_2507_21433_amd import binding as rc
from paper_2507_21433_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def buffers(w, pr):
    L, P, Q = w.L, w.P, w.Q
    nshape = (L, Q) if w.mode == 0 else (L, Q, w.H)
    b = dict(qk=torch.empty(nshape, dtype=torch.float32, device=DEV), qv=torch.empty(nshape, dtype=torch.float32, device=DEV),
             ws_match=torch.empty(rc.rc_match_workspace_size(pr["kq"], w.mode, Q, P), dtype=torch.uint8, device=DEV),
             ws_remap=torch.empty(rc.rc_remap_workspace_size(L, w.R, w.E, Q, w.NB), dtype=torch.uint8, device=DEV),
             ws_lm=torch.empty(max(16, rc.rc_layer_mean_workspace_size(pr["kq"], Q, P)), dtype=torch.uint8, device=DEV),
             ws_pat=torch.empty(rc.lib().rc_pat_workspace_size(), dtype=torch.uint8, device=DEV),
             match=dict(best_idx=torch.empty((L, Q), dtype=torch.int32, device=DEV),
                        best_score=torch.empty((L, Q), dtype=torch.float32, device=DEV),
                        match_idx=torch.empty((L, Q), dtype=torch.int32, device=DEV),
                        second_score=torch.empty((L, Q), dtype=torch.float32, device=DEV)),
             remap=dict(tables=torch.empty_like(pr["tables"]), refcount=torch.empty_like(pr["refcount"]),
                        freed=torch.empty((L, Q), dtype=torch.uint8, device=DEV),
                        n_remapped=torch.empty((L,), dtype=torch.int32, device=DEV)),
             lm=dict(best_idx=torch.empty((Q,), dtype=torch.int32, device=DEV),
                     best_dist=torch.empty((Q,), dtype=torch.float32, device=DEV),
                     match_idx=torch.empty((Q,), dtype=torch.int32, device=DEV),
                     second_dist=torch.empty((Q,), dtype=torch.float32, device=DEV)),
             pat=dict(threshold=torch.empty(1, dtype=torch.float32, device=DEV),
                      n_finite=torch.empty(1, dtype=torch.int64, device=DEV)),
             decided=torch.empty((Q,), dtype=torch.int32, device=DEV))
    return b


def step(w, pr, pk, pv, lv, b):
    rc.rc_block_norms(pr["kq"], pr["vq"], w.mode, b["qk"], b["qv"])
    rc.rc_match_blocks(pr["kq"], pr["vq"], b["qk"], b["qv"], pr["kp"], pr["vp"], pk, pv, pr["live"], w.tau, w.mode,
                       workspace=b["ws_match"], out=b["match"])
    rc.rc_remap_block_table(pr["tables"], pr["query_ids"], None, b["match"]["match_idx"], w.P, w.NB, pr["refcount"],
                            workspace=b["ws_remap"], out=b["remap"])
    if w.mode == 0:
        rc.rc_match_blocks_layer_mean(pr["kq"], pr["vq"], b["qk"], b["qv"], pr["kp"], pr["vp"], pk, pv, lv, float("inf"),
                                      workspace=b["ws_lm"], out=b["lm"])
        rc.rc_pat_threshold(b["lm"]["best_dist"], 50.0, workspace=b["ws_pat"], out=b["pat"])
        rc.rc_apply_threshold(b["lm"]["best_idx"], b["lm"]["best_dist"], b["pat"]["threshold"], b["decided"])


def flat(b, mode):
    """Every buffer the step writes (the layer-mean part only runs in block mode)."""
    out = []
    for k in ("match", "remap") + (("lm", "pat") if mode == 0 else ()):
        out += [b[k][n] for n in sorted(b[k])]
    return out + ([b["decided"]] if mode == 0 else []) + [b["qk"], b["qv"]]


# (the last case has 19 rounds of tiles: the launch whose tile schedule lives in words that a kernel clears first)
@pytest.mark.parametrize("wl,kw", [(1, {}), (2, dict(L=3, P=700, Q=300, R=4, E=260)), (5, dict(L=2, P=300, Q=40, R=1, E=340)),
                                   (2, dict(L=260, P=513, Q=1300, H=1, R=1, E=1813))])
def test_step_in_a_graph(wl, kw):
    w = synth.scaled(synth.WORKLOADS[wl], name=f"graph_cfg{wl}", **kw)
    say(f"{w.name}: L={w.L} P={w.P} Q={w.Q} mode={w.mode}")
    pr = synth.make_problem(w, DEV)
    pk, pv = rc.rc_block_norms(pr["kp"], pr["vp"], w.mode)
    lv = pr["live"].min(dim=0).values.contiguous()
    eager, graphed = buffers(w, pr), buffers(w, pr)
    step(w, pr, pk, pv, lv, eager)
    step(w, pr, pk, pv, lv, graphed)          # warm-up on the capture buffers, outside the graph
    torch.cuda.synchronize()
    want = [t.clone() for t in flat(eager, w.mode)]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(w, pr, pk, pv, lv, graphed)
    for replay in range(4):
        for t in flat(graphed, w.mode):
            t.zero_() if t.dtype != torch.float32 else t.fill_(float("nan"))
        step(w, pr, pk, pv, lv, eager)        # the program's own eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b_ in zip(flat(graphed, w.mode), want):
            assert torch.equal(a.view(torch.uint8) if a.dtype == torch.float32 else a,
                               b_.view(torch.uint8) if b_.dtype == torch.float32 else b_), f"replay {replay} differs"
    say(f"{w.name}: 4 replays identical to the eager step")
