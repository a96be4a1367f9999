"""Parity of rc_pat_threshold / rc_apply_threshold (percentile-based adaptive thresholding) with the CPU oracle:
the threshold is an exact order statistic, so everything here is bit-exact.  Needs a real MI355X."""
import sys

import numpy as np
import pytest
import torch

from paper_2507_21433_amd import binding as rc
from paper_2507_21433_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def gpu_pat(s, p):
    out = rc.rc_pat_threshold(torch.as_tensor(s, device=DEV), p)
    torch.cuda.synchronize()
    return out["threshold"].cpu().numpy()[0], int(out["n_finite"].cpu()[0])


def same(a, b):
    return (a == b) or (np.isnan(a) and np.isnan(b))


@pytest.mark.parametrize("n", [1, 2, 5, 255, 256, 257, 4097, 100003, 3_000_001])
def test_pat_random(oracle, n):
    say(f"pat n={n}")
    rng = np.random.RandomState(n % 1000)
    # the distance mix of a workload: a cluster of near-duplicates, a cluster of fresh blocks, ties, and no-candidate entries
    s = np.where(rng.rand(n) < 0.3, 0.15 + 0.01 * rng.randn(n), 1.41 + 0.005 * rng.randn(n)).astype(np.float32)
    s[rng.rand(n) < 0.05] = np.float32(0.15)
    s[rng.rand(n) < 0.02] = np.inf
    for p in (0.0, 0.1, 20.0, 33.3, 50.0, 80.0, 99.5, 100.0):
        t, c = gpu_pat(s, p)
        to, co = oracle.pat_threshold(s, p)
        assert c == co and same(t, to), (n, p, t, to)


def test_pat_special_values(oracle):
    say("pat: signs, zeros, denormals, huge values, all equal, nothing finite")
    rng = np.random.RandomState(4)
    cases = [
        np.array([-3, 2, -1, 0, 5, -7, 1e-42, -1e-42, 3e38, -3e38], dtype=np.float32),
        np.full(1000, 0.25, dtype=np.float32),
        np.array([np.inf, np.nan, -np.inf], dtype=np.float32),
        (rng.randn(5000) * 10.0 ** rng.randint(-30, 30, 5000)).astype(np.float32),
        np.arange(70000, dtype=np.float32)[::-1].copy(),
    ]
    for s in cases:
        for p in (0.0, 10.0, 33.3, 50.0, 80.0, 100.0):
            t, c = gpu_pat(s, p)
            to, co = oracle.pat_threshold(s, p)
            assert c == co and (same(t, to) or (t == 0 and to == 0)), (s[:4], p, t, to)
    t, c = gpu_pat(np.zeros(0, dtype=np.float32), 80.0)
    assert np.isneginf(t) and c == 0
    with pytest.raises(rc.RcError) as e:
        rc.rc_pat_threshold(torch.zeros(4, device=DEV), 101.0)
    assert e.value.code == 1


def test_pat_rank_comes_from_the_callers_double(oracle):
    """p = 0.1 of 1000 samples is rank ceil(1.0) = 1; the same p rounded to float (0.100000001...) would give rank 2."""
    say("pat: p = 0.1, n = 1000 (rank 1 in double, 2 if p were rounded to float)")
    s = np.random.RandomState(8).permutation(1000).astype(np.float32) + 5
    t, c = gpu_pat(s, 0.1)
    to, co = oracle.pat_threshold(s, 0.1)
    assert c == co == 1000 and t == to == 5.0
    assert oracle.pat_threshold(s, float(np.float32(0.1)))[0] == 6.0      # what the float ABI used to compute


def test_apply_threshold(oracle):
    say("apply threshold")
    rng = np.random.RandomState(6)
    n = 10007
    idx = rng.randint(-1, 50, n).astype(np.int32)
    d = np.abs(rng.randn(n)).astype(np.float32)
    d[idx < 0] = np.inf
    d[::97] = np.nan
    for thr in (np.float32(0.7), d[5], np.float32(-np.inf), np.float32(np.inf)):
        g = rc.rc_apply_threshold(torch.as_tensor(idx, device=DEV), torch.as_tensor(d, device=DEV),
                                  torch.tensor([thr], dtype=torch.float32, device=DEV))
        torch.cuda.synchronize()
        assert np.array_equal(g.cpu().numpy(), oracle.apply_threshold(idx, d, thr))


def test_pat_end_to_end(oracle):
    # warm-up steps with sharing disabled collect the best distances, the percentile becomes the threshold of the
    # next step; the oracle runs the same protocol on its own distances
    say("pat end to end: 3 warm-up steps, then a decided step")
    ws = [synth.scaled(synth.WORKLOADS[2], name=f"pat_step{i}", L=2, P=300, Q=48, planted_frac=0.4, R=1, E=348, seed=60 + i)
          for i in range(4)]
    g_samples, o_samples = [], []
    for w in ws[:3]:
        pr = synth.make_problem(w, DEV)
        qk, qv = rc.rc_block_norms(pr["kq"], pr["vq"], 0)
        pk, pv = rc.rc_block_norms(pr["kp"], pr["vp"], 0)
        lv = pr["live"].min(dim=0).values.contiguous()
        g = rc.rc_match_blocks_layer_mean(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, lv, float("-inf"))
        assert (g["match_idx"] == -1).all()                      # reuse is off while warming up
        g_samples.append(g["best_dist"])
        o = oracle.layer_mean(0, *(synth.bits(pr[n]) for n in ("kq", "vq", "kp", "vp")), lv.cpu().numpy(), -np.inf)
        assert (o["match_idx"] == -1).all()
        o_samples.append(o["best_dist"])
    gs = torch.cat(g_samples)
    for p, frac in ((20.0, 0.2), (80.0, 0.8), (100.0, 1.0)):
        thr = rc.rc_pat_threshold(gs, p)
        # bit-exact against the oracle's selection on the very same samples
        to, _ = oracle.pat_threshold(gs.cpu().numpy(), p)
        assert thr["threshold"].cpu().numpy()[0] == to
        # and close to the oracle's own protocol (its samples differ from the GPU's by rounding only)
        to2, _ = oracle.pat_threshold(np.concatenate(o_samples).astype(np.float32), p)
        assert abs(float(to) - float(to2)) <= 2e-3
        assert abs((gs <= thr["threshold"]).float().mean().item() - frac) <= 1.0 / gs.numel() + 1e-6
        # the decided step
        w = ws[3]
        pr = synth.make_problem(w, DEV)
        qk, qv = rc.rc_block_norms(pr["kq"], pr["vq"], 0)
        pk, pv = rc.rc_block_norms(pr["kp"], pr["vp"], 0)
        lv = pr["live"].min(dim=0).values.contiguous()
        g = rc.rc_match_blocks_layer_mean(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, lv, float("inf"))
        m = rc.rc_apply_threshold(g["best_idx"], g["best_dist"], thr["threshold"])
        torch.cuda.synchronize()
        want = oracle.apply_threshold(g["best_idx"].cpu().numpy(), g["best_dist"].cpu().numpy(), to)
        assert np.array_equal(m.cpu().numpy(), want)
        if p == 100.0:
            # the largest warm-up distance accepts (nearly) everything: fresh blocks sit at ~1.41 with a spread of 1e-3
            assert (m >= 0).float().mean().item() > 0.5
        if p == 20.0:
            plan = pr["plan"]
            assert set(np.flatnonzero(m.cpu().numpy() >= 0)) <= set(plan.planted_slots.tolist())
