#!/usr/bin/env python3
"""Benchmark of the reusable-KV-block search on one MI355X.

A step is one pass of the whole hot path over one batch of new blocks, all layers:
  rc_block_norms(query blocks) -> rc_match_blocks(queries x resident pool) -> rc_remap_block_table
with the pool's squared norms cached from when the blocks were sealed (the paper's
Stage 2 computes a block's norms once and reuses them).  Inputs are resident in HBM
before the timed region.  Prints ONE JSON line.

The headline (`value`, `roofline`, `cpu_baseline`, `kernels`) is the largest workload of the
benchmark definition that fits one GPU, cfg4 (210 GB of KV); the `configs` object carries the
same step, timed the same way in the same run, for every one of the five workloads.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f16": 2500.0, "bf16": 2500.0}   # dense MFMA, MI355X
PEAK_HBM_GBS = 8000.0
# HBM bytes per launch of the tile kernel, per workload, from rocprofv3 counter runs of this script
# (FETCH_SIZE and WRITE_SIZE, scaled by what the same counters read for the 1 GiB copy issued below).
# The table names the kernel source it was measured on; it is ignored when that source has changed.
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
KERNEL_SOURCES = ("paper_2507_21433_amd/csrc/rc_match.hip", "paper_2507_21433_amd/csrc/rc_common.hpp")


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def kernel_source_hash():
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def load_traffic():
    """{workload name: HBM bytes per launch} if the tracked table matches the kernel source, else ({}, reason)."""
    try:
        with open(TRAFFIC_TABLE) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return {}, "profiles/hbm_traffic.json is missing"
    if t.get("kernel_source_sha256") != kernel_source_hash():
        return {}, "profiles/hbm_traffic.json was measured on another version of the kernel source"
    return {k: v["hbm_bytes_per_launch"] for k, v in t.get("workloads", {}).items()}, None


def cpu_baseline(w, pr, budget, one_core):
    """The oracle as it stands, timed on the host cores on a bounded sample of the workload: whole layers
    while they fit a budget of pairs, else the first queries of the first layer."""
    from oracle import rc_oracle
    from paper_2507_21433_amd import synth
    rc_oracle.build()
    if w.mode != 0:
        budget = budget / 4             # the per-head search costs about four times as much per pair
    per_layer = w.P * w.Q
    if per_layer <= budget:
        n_layers, n_q = int(max(1, min(w.L, budget // per_layer))), w.Q
    else:
        n_layers, n_q = 1, int(max(1, budget // w.P))
    a = [synth.bits(pr[n][:n_layers, :n_q] if n[1] == "q" else pr[n][:n_layers]) for n in ("kq", "vq", "kp", "vp")]
    live = pr["live"][:n_layers].cpu().numpy()
    t0 = time.time()
    rc_oracle.match(0 if w.dtype == "f16" else 1, w.mode, *a, live, w.tau)
    dt = time.time() - t0
    pairs = n_layers * w.P * n_q
    res = {"value": pairs / dt, "unit": "pairs/s", "cores": rc_oracle.n_threads(), "kind": "oracle",
           "sample": f"rc_oracle.match on the first {n_q} of {w.Q} query blocks of the first {n_layers} of {w.L} layers "
                     f"of {w.name} ({pairs} pairs, {dt:.1f} s)"}
    if one_core:
        # the same oracle on one core, on a sixteenth of the sample (the first layer, fewer queries)
        try:
            import ctypes
            gomp = ctypes.CDLL("libgomp.so.1")
            n1 = int(max(1, min(n_q, pairs // 16 // w.P)))
            a1 = [x[:1, :n1] if i < 2 else x[:1] for i, x in enumerate(a)]
            gomp.omp_set_num_threads(1)
            t0 = time.time()
            rc_oracle.match(0 if w.dtype == "f16" else 1, w.mode, *a1, live[:1], w.tau)
            dt1 = time.time() - t0
            gomp.omp_set_num_threads(rc_oracle.n_threads())
            res["one_core_value"] = w.P * n1 / dt1
            res["one_core_sample"] = f"first {n1} query blocks of the first layer ({w.P * n1} pairs, {dt1:.1f} s)"
        except OSError:
            pass
    return res


def timed(torch, fn, reps):
    """Average milliseconds of fn() over reps calls, by events on the stream the kernels are launched on."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def run_config(args, w, traffic, extras, cpu_budget):
    """The step on one workload; with `extras` also the entry points that are timed beside it."""
    import torch
    from paper_2507_21433_amd import binding as rc
    from paper_2507_21433_amd import synth
    dev = "cuda:0"
    log(f"workload {w.name}: L={w.L} P={w.P} Q={w.Q} T={w.T} dtype={w.dtype} mode={w.mode}")
    t0 = time.time()
    pr = synth.make_problem(w, dev)
    torch.cuda.synchronize()
    log(f"inputs resident ({(w.L * (w.P + w.Q) * w.block_bytes) / 1e9:.1f} GB of KV) after {time.time() - t0:.1f} s")

    L, P, Q = w.L, w.P, w.Q
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    # pool norms: computed when the blocks were sealed, cached since (also timed once, as the cold fill)
    pk, pv = rc.rc_block_norms(pr["kp"], pr["vp"], w.mode)
    torch.cuda.synchronize()
    e0.record()
    rc.rc_block_norms(pr["kp"], pr["vp"], w.mode, pk, pv)
    e1.record()
    torch.cuda.synchronize()
    pool_norm_ms = e0.elapsed_time(e1)

    nshape = (L, Q) if w.mode == 0 else (L, Q, w.H)
    qk = torch.empty(nshape, dtype=torch.float32, device=dev)
    qv = torch.empty(nshape, dtype=torch.float32, device=dev)
    ws_match = torch.empty(rc.rc_match_workspace_size(pr["kq"], w.mode, Q, P), dtype=torch.uint8, device=dev)
    ws_remap = torch.empty(rc.rc_remap_workspace_size(L, w.R, w.E, Q, w.NB), dtype=torch.uint8, device=dev)
    out = dict(best_idx=torch.empty((L, Q), dtype=torch.int32, device=dev),
               best_score=torch.empty((L, Q), dtype=torch.float32, device=dev),
               match_idx=torch.empty((L, Q), dtype=torch.int32, device=dev),
               second_score=torch.empty((L, Q), dtype=torch.float32, device=dev))
    remap_out = dict(tables=torch.empty_like(pr["tables"]), refcount=torch.empty_like(pr["refcount"]),
                     freed=torch.empty((L, Q), dtype=torch.uint8, device=dev),
                     n_remapped=torch.empty((L,), dtype=torch.int32, device=dev))

    def step(ev=None):
        if ev:
            ev[0].record()
        rc.rc_block_norms(pr["kq"], pr["vq"], w.mode, qk, qv)
        if ev:
            ev[1].record()
        rc.rc_match_blocks(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, pr["live"], w.tau, w.mode,
                           workspace=ws_match, out=out)
        if ev:
            ev[2].record()
        res = rc.rc_remap_block_table(pr["tables"], pr["query_ids"], None, out["match_idx"], P, w.NB, pr["refcount"],
                                      workspace=ws_remap, out=remap_out)
        if ev:
            ev[3].record()
        return res

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        res = step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    norm_ms = sum(e[0].elapsed_time(e[1]) for e in events) / args.steps
    match_ms = sum(e[1].elapsed_time(e[2]) for e in events) / args.steps
    remap_ms = sum(e[2].elapsed_time(e[3]) for e in events) / args.steps

    pairs = L * P * Q
    flop = pairs * 4.0 * w.D                       # 2 (mul+add) x D x 2 (K and V) per pair
    kv_bytes = L * (P + Q) * w.block_bytes         # every pool and query block read once
    match_tflops = flop / (match_ms * 1e-3) / 1e12
    match_gbs = kv_bytes / (match_ms * 1e-3) / 1e9
    # which roof binds: the launch's FLOP per byte of KV against the ridge of the two peaks (312 FLOP/byte)
    intensity = flop / kv_bytes if kv_bytes else 0.0
    ridge = PEAK_TFLOPS[w.dtype] * 1e12 / (PEAK_HBM_GBS * 1e9)
    roofline = {"kernel": "match_tile_kernel (inside rc_match_blocks)"}
    if intensity >= ridge:
        roofline.update(bound="mfma", achieved=match_tflops, peak=PEAK_TFLOPS[w.dtype], unit="TFLOP/s",
                        frac=match_tflops / PEAK_TFLOPS[w.dtype])
    else:
        roofline.update(bound="hbm", achieved=match_gbs, peak=PEAK_HBM_GBS, unit="GB/s", frac=match_gbs / PEAK_HBM_GBS)
    roofline.update(traffic=traffic.get(w.name) if not args.layers else None,
                    algorithmic_bytes=kv_bytes, algorithmic_flop=flop, flop_per_byte=intensity, ridge_flop_per_byte=ridge,
                    tflops=match_tflops, mfma_frac=match_tflops / PEAK_TFLOPS[w.dtype],
                    gb_per_s=match_gbs, hbm_frac=match_gbs / PEAK_HBM_GBS)
    qnorm_bytes = L * Q * w.block_bytes
    remap_bytes = L * (2 * w.R * w.E * 4 + 2 * w.NB * 4)
    kernels = {
        "rc_match_blocks": {"ms": match_ms, "tflops": match_tflops, "kv_gb_per_s": match_gbs,
                            "hbm_frac": match_gbs / PEAK_HBM_GBS,
                            "flop_per_byte": flop / kv_bytes},
        "rc_block_norms(queries)": {"ms": norm_ms, "gb_per_s": qnorm_bytes / (norm_ms * 1e-3) / 1e9,
                                    "hbm_frac": qnorm_bytes / (norm_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
        "rc_block_norms(pool, cold fill, not in the step)": {
            "ms": pool_norm_ms, "gb_per_s": L * P * w.block_bytes / (pool_norm_ms * 1e-3) / 1e9,
            "hbm_frac": L * P * w.block_bytes / (pool_norm_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
        "rc_remap_block_table": {"ms": remap_ms, "gb_per_s": remap_bytes / (remap_ms * 1e-3) / 1e9,
                                 "hbm_frac": remap_bytes / (remap_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
    }
    streaming = None
    errors = {}
    if extras:
        try:
            streaming = run_extras(args, w, pr, kernels, dict(qk=qk, qv=qv, pk=pk, pv=pv, out=out, flop=flop, kv_bytes=kv_bytes,
                                                              pairs=pairs))
        except Exception as e:   # noqa: BLE001  (the measurements beside the step must not take the step's figures with them)
            log(f"measurements beside the step failed: {e!r}")
            errors["measurements beside the step"] = repr(e)
            torch.cuda.empty_cache()
    matched = int((out["match_idx"] >= 0).sum().item())
    n_remapped = int(res["n_remapped"].sum().item())

    cpu = None
    if cpu_budget > 0:
        log("timing the CPU oracle on the host cores ...")
        cpu = cpu_baseline(w, pr, cpu_budget, one_core=extras)

    block = {
        "value": pairs / (ms_step * 1e-3), "unit": "pairs/s", "ms_per_step": ms_step, "dtype": w.dtype,
        "config": {"workload": w.name, "layers": L, "pool_blocks_per_layer": P, "query_blocks_per_layer": Q,
                   "block_tokens": w.T, "kv_heads": w.H, "head_dim": w.Dh, "mode": "block" if w.mode == 0 else "per_head_all",
                   "tau": w.tau, "tables": [w.R, w.E], "pool_norms": "cached"},
        "kv_gb_per_s": kv_bytes / (ms_step * 1e-3) / 1e9,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
        "matched_queries": matched, "remapped_entries": n_remapped,
    }
    if extras:
        block["streaming"] = streaming
    if errors:
        block["side_errors"] = errors
    del pr, pk, pv, qk, qv, ws_match, ws_remap, out, remap_out
    torch.cuda.empty_cache()
    return block


def run_extras(args, w, pr, kernels, s):
    """Entry points timed beside the step (not part of it); fills `kernels`, returns the streaming object."""
    import torch
    from paper_2507_21433_amd import binding as rc
    dev = "cuda:0"
    L, P, Q = w.L, w.P, w.Q
    qk, qv, pk, pv, out, flop, kv_bytes, pairs = (s[k] for k in ("qk", "qv", "pk", "pv", "out", "flop", "kv_bytes", "pairs"))
    if L > 1 and P > 0:
        # the same search called for one layer at a time, as an engine that scores a layer when its KV is written
        # would call it: few tiles, so every tile's reduction is split over several workgroups
        one = [pr[n][:1] for n in ("kq", "vq", "kp", "vp")]
        qk1, qv1, pk1, pv1 = qk[:1], qv[:1], pk[:1], pv[:1]
        live1 = pr["live"][:1]
        ws1 = torch.empty(rc.rc_match_workspace_size(one[0], w.mode, Q, P), dtype=torch.uint8, device=dev)
        out1 = {k: torch.empty_like(v[:1]) for k, v in out.items()}
        one_ms = timed(torch, lambda: rc.rc_match_blocks(one[0], one[1], qk1, qv1, one[2], one[3], pk1, pv1, live1, w.tau,
                                                         w.mode, workspace=ws1, out=out1), args.steps)
        kernels["rc_match_blocks(one layer per call, not in the step)"] = {
            "ms": one_ms, "tflops": flop / L / (one_ms * 1e-3) / 1e12, "workspace_bytes": ws1.numel()}
        del ws1
    if args.candidates > 0 and P > 0:
        # candidate-restricted Stage 2 (not part of the step): C random pool blocks per query, timed the same way
        C = args.candidates
        gen = torch.Generator(device=dev)
        gen.manual_seed(12345)
        cand = torch.randint(0, P, (L, Q, C), generator=gen, device=dev, dtype=torch.int32)
        cout = rc.rc_score_candidates(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, pr["live"], cand, w.tau, w.mode)
        cand_ms = timed(torch, lambda: rc.rc_score_candidates(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv,
                                                              pr["live"], cand, w.tau, w.mode, out=cout), args.steps)
        cand_bytes = L * Q * C * w.block_bytes       # one pool block per listed pair; the query block stays in the L2
        kernels[f"rc_score_candidates(C={C}, not in the step)"] = {
            "ms": cand_ms, "gb_per_s": cand_bytes / (cand_ms * 1e-3) / 1e9,
            "hbm_frac": cand_bytes / (cand_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "pairs_per_s": L * Q * C / (cand_ms * 1e-3)}
        # Stage 2 as the paper runs it: layer-mean distance of C listed pairs per query, one list for all layers
        gen.manual_seed(54321)
        cand1 = torch.randint(0, P, (Q, C), generator=gen, device=dev, dtype=torch.int32)
        lv1 = pr["live"].min(dim=0).values.contiguous()
        cdo = rc.rc_candidate_distances(pr["kq"], pr["vq"], pr["kp"], pr["vp"], lv1, cand1, 0.5)
        ws_cd = torch.empty(max(16, rc.lib().rc_candidate_distances_workspace_size(rc.ctypes.byref(rc.kv_desc(pr["kq"])), Q, C)),
                            dtype=torch.uint8, device=dev)
        cd_ms = timed(torch, lambda: rc.rc_candidate_distances(pr["kq"], pr["vq"], pr["kp"], pr["vp"], lv1, cand1, 0.5,
                                                               workspace=ws_cd, out=cdo), args.steps)
        cd_bytes = L * Q * C * w.block_bytes
        kernels[f"rc_candidate_distances(C={C}, not in the step)"] = {
            "ms": cd_ms, "gb_per_s": cd_bytes / (cd_ms * 1e-3) / 1e9,
            "hbm_frac": cd_bytes / (cd_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "pairs_per_s": Q * C / (cd_ms * 1e-3)}
        del cand, cout, cdo, ws_cd
    if args.layer_mean and P > 0 and w.mode == 0:
        # the paper's own measure (not part of the step): layer-mean Euclidean distance, one decision per block
        lv = pr["live"].min(dim=0).values.contiguous()
        ws_lm = torch.empty(max(16, rc.rc_layer_mean_workspace_size(pr["kq"], Q, P)), dtype=torch.uint8, device=dev)
        lm = rc.rc_match_blocks_layer_mean(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, lv, 0.5, workspace=ws_lm)
        lm_ms = timed(torch, lambda: rc.rc_match_blocks_layer_mean(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, lv,
                                                                   0.5, workspace=ws_lm, out=lm), max(2, args.steps // 2))
        kernels["rc_match_blocks_layer_mean(not in the step)"] = {
            "ms": lm_ms, "tflops": flop / (lm_ms * 1e-3) / 1e12, "mfma_frac": flop / (lm_ms * 1e-3) / 1e12 / PEAK_TFLOPS[w.dtype],
            "kv_gb_per_s": kv_bytes / (lm_ms * 1e-3) / 1e9, "workspace_bytes": ws_lm.numel(),
            "matched_blocks": int((lm["match_idx"] >= 0).sum().item())}
        del ws_lm, lm
        if L > 1:
            # the same search called for one layer (few tiles: every tile's reduction is split over several workgroups)
            one = [pr[n][:1] for n in ("kq", "vq", "kp", "vp")]
            ws1 = torch.empty(max(16, rc.rc_layer_mean_workspace_size(one[0], Q, P)), dtype=torch.uint8, device=dev)
            lm1 = rc.rc_match_blocks_layer_mean(one[0], one[1], qk[:1], qv[:1], one[2], one[3], pk[:1], pv[:1], lv, 0.5,
                                                workspace=ws1)
            lm1_ms = timed(torch, lambda: rc.rc_match_blocks_layer_mean(one[0], one[1], qk[:1], qv[:1], one[2], one[3], pk[:1],
                                                                        pv[:1], lv, 0.5, workspace=ws1, out=lm1), args.steps)
            kernels["rc_match_blocks_layer_mean(one layer per call, not in the step)"] = {
                "ms": lm1_ms, "tflops": flop / L / (lm1_ms * 1e-3) / 1e12, "workspace_bytes": ws1.numel()}
            del ws1, lm1
    if args.pat_samples > 0:
        # percentile threshold over a warm-up sample of this many distances (not part of the step)
        n = args.pat_samples
        gen = torch.Generator(device=dev)
        gen.manual_seed(777)
        smp = torch.where(torch.rand(n, generator=gen, device=dev) < 0.3,
                          0.15 + 0.01 * torch.randn(n, generator=gen, device=dev),
                          1.41 + 0.005 * torch.randn(n, generator=gen, device=dev)).contiguous()
        ws_pat = torch.empty(rc.lib().rc_pat_workspace_size(), dtype=torch.uint8, device=dev)
        po = rc.rc_pat_threshold(smp, 80.0, workspace=ws_pat)
        pat_ms = timed(torch, lambda: rc.rc_pat_threshold(smp, 80.0, workspace=ws_pat, out=po), args.steps)
        kernels[f"rc_pat_threshold(n={n}, p=80, not in the step)"] = {
            "ms": pat_ms, "gb_per_s": 4.0 * n / (pat_ms * 1e-3) / 1e9, "threshold": float(po["threshold"].item())}
    if args.admit and P >= 2 * Q and w.mode == 0:
        # streaming pool maintenance (not part of the step): the last Q slots are declared free and every query of
        # the step that no layer matched is admitted there (K, V and norms of all layers are copied)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        live1 = pr["live"].min(dim=0).values.contiguous()
        live1[P - Q:] = 0
        none = (out["match_idx"] >= 0).sum(dim=0).eq(0)
        m1 = torch.where(none, torch.full((Q,), -1, dtype=torch.int32, device=dev), torch.zeros(Q, dtype=torch.int32, device=dev))
        live_w = live1.clone()
        ws_ad = torch.empty(max(16, rc.lib().rc_pool_admit_workspace_size(Q, P)), dtype=torch.uint8, device=dev)
        ao = rc.rc_pool_admit(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, live_w, m1, workspace=ws_ad)
        torch.cuda.synchronize()
        n_adm = int(ao["n_admitted"].item())
        ad_ms = 0.0
        for _ in range(args.steps):
            live_w.copy_(live1)
            e0.record()
            rc.rc_pool_admit(pr["kq"], pr["vq"], qk, qv, pr["kp"], pr["vp"], pk, pv, live_w, m1, workspace=ws_ad, out=ao)
            e1.record()
            torch.cuda.synchronize()
            ad_ms += e0.elapsed_time(e1) / args.steps
        ad_bytes = 2.0 * n_adm * L * w.block_bytes        # every admitted block read once and written once
        kernels["rc_pool_admit(not in the step)"] = {
            "ms": ad_ms, "admitted_blocks": n_adm, "gb_per_s": ad_bytes / (ad_ms * 1e-3) / 1e9,
            "hbm_frac": ad_bytes / (ad_ms * 1e-3) / 1e9 / PEAK_HBM_GBS}
    streaming = None
    torch.cuda.empty_cache()
    stream_bytes = args.streaming * L * Q * w.block_bytes + (4 << 30)   # the steps' inputs plus temporaries while drawing them
    if args.streaming > 0 and w.mode == 0 and P >= (args.streaming + 1) * Q and torch.cuda.mem_get_info()[0] > stream_bytes + (8 << 30):
        # the paper's steady state (not the timed step above): consecutive decoding steps over a pool that is FULL,
        # with the paper's own measure.  Per step: norms of the new blocks, layer-mean search, decision against a
        # threshold that lives on the device, remap of a layer-shared table with reference counts, last-use stamps of
        # the partners, the references of the requests that end at this step are dropped, the unreferenced blocks
        # leave the pool in LRU order to make room, admission of the blocks that found no partner, their metadata.
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        S = args.streaming
        lv = torch.ones(P, dtype=torch.uint8, device=dev)            # every slot holds a resident block
        thr_dev = torch.full((1,), 0.5, dtype=torch.float32, device=dev)
        gen = torch.Generator(device=dev)
        gen.manual_seed(4242)
        n_copy = int(0.3 * Q)
        steps_kq, steps_vq = [], []
        for sidx in range(S):                                         # inputs of every step, built before the clock starts
            kq_s = torch.empty_like(pr["kq"])
            vq_s = torch.empty_like(pr["vq"])
            tgt = torch.randint(S * Q, P, (n_copy,), generator=gen, device=dev)   # copies of blocks that stay referenced
            for l in range(L):                                        # layer by layer: the fp32 temporaries stay small
                kq_s[l] = torch.randn(pr["kq"].shape[1:], generator=gen, device=dev, dtype=torch.float32).to(pr["kq"].dtype)
                vq_s[l] = torch.randn(pr["vq"].shape[1:], generator=gen, device=dev, dtype=torch.float32).to(pr["vq"].dtype)
                kq_s[l, :n_copy] = (pr["kp"][l, tgt].float() + w.sigma * torch.randn((n_copy,) + tuple(pr["kp"].shape[2:]), generator=gen, device=dev)).to(pr["kq"].dtype)
                vq_s[l, :n_copy] = (pr["vp"][l, tgt].float() + w.sigma * torch.randn((n_copy,) + tuple(pr["vp"].shape[2:]), generator=gen, device=dev)).to(pr["vq"].dtype)
            steps_kq.append(kq_s)
            steps_vq.append(vq_s)
        ws_lm2 = torch.empty(max(16, rc.rc_layer_mean_workspace_size(pr["kq"], Q, P)), dtype=torch.uint8, device=dev)
        ws_ad2 = torch.empty(max(16, rc.lib().rc_pool_admit_workspace_size(Q, P)), dtype=torch.uint8, device=dev)
        ws_rm2 = torch.empty(rc.rc_remap_workspace_size(1, 1, Q, Q, P + Q), dtype=torch.uint8, device=dev)
        table = (P + torch.arange(Q, dtype=torch.int32, device=dev)).reshape(1, 1, Q).contiguous()
        qids = (P + torch.arange(Q, dtype=torch.int32, device=dev)).contiguous()
        refc = torch.ones((1, P + Q), dtype=torch.int32, device=dev)  # every resident block is referenced once
        refc_out = torch.empty_like(refc)
        stamp = torch.zeros(P, dtype=torch.int32, device=dev)
        # the requests that end at step s hold the blocks of slots [s*Q, (s+1)*Q)
        ending = [torch.arange(sidx * Q, (sidx + 1) * Q, dtype=torch.int32, device=dev) for sidx in range(S)]
        lm2, ad2, ev2 = None, None, None
        rm2 = dict(tables=torch.empty_like(table), refcount=refc_out, freed=torch.empty((1, Q), dtype=torch.uint8, device=dev),
                   n_remapped=torch.empty((1,), dtype=torch.int32, device=dev))
        dec = torch.empty((Q,), dtype=torch.int32, device=dev)
        shared, admitted, evicted = [], [], []
        torch.cuda.synchronize()
        e0.record()
        for sidx in range(S):
            rc.rc_block_norms(steps_kq[sidx], steps_vq[sidx], 0, qk, qv)
            lm2 = rc.rc_match_blocks_layer_mean(steps_kq[sidx], steps_vq[sidx], qk, qv, pr["kp"], pr["vp"], pk, pv, lv,
                                                float("inf"), workspace=ws_lm2, out=lm2)
            rc.rc_apply_threshold(lm2["best_idx"], lm2["best_dist"], thr_dev, dec)
            rc.rc_remap_block_table(table, qids, None, dec.reshape(1, Q), P, P + Q, refc, workspace=ws_rm2, out=rm2)
            pool_refc = refc_out[0, :P]                                # (a view: the first P counts are the pool's slots)
            rc.rc_pool_touch(dec, sidx + 1, stamp)
            rc.rc_refcount_release(ending[sidx], pool_refc)
            ev2 = rc.rc_pool_evict(lv, pool_refc, stamp, dec, out=ev2)
            ad2 = rc.rc_pool_admit(steps_kq[sidx], steps_vq[sidx], qk, qv, pr["kp"], pr["vp"], pk, pv, lv, dec,
                                   workspace=ws_ad2, out=ad2)
            rc.rc_pool_touch(ad2["slot_of_query"], sidx + 1, stamp)
            rc.rc_pool_touch(ad2["slot_of_query"], 1, pool_refc)
            refc[0, :P].copy_(pool_refc)                               # the counts carry over; the new ids start at 1 again
            shared.append((dec >= 0).sum())
            admitted.append(ad2["n_admitted"].clone())
            evicted.append(ev2["n_evicted"].clone())
        e1.record()
        torch.cuda.synchronize()
        st_ms = e0.elapsed_time(e1) / S
        streaming = {"steps": S, "ms_per_step": st_ms, "pairs_per_s": pairs / (st_ms * 1e-3),
                     "pool": "full: every slot live and referenced; the requests that end free Q blocks per step",
                     "shared_per_step": [int(x.item()) for x in shared],
                     "evicted_per_step": [int(x.item()) for x in evicted],
                     "admitted_per_step": [int(x.item()) for x in admitted],
                     "live_slots_at_the_end": int(lv.sum().item()), "pool_slots": P,
                     "what": "norms(Q) + layer-mean search + device-threshold decision + layer-shared remap + last-use stamps + "
                             "release of ended requests + LRU eviction of unreferenced blocks + admission"}
    return streaming


def mfma_probe():
    """What this machine sustains on back-to-back fp16 MFMA with random operands and nothing else (the chip lowers its
    clock under matrix load): TFLOP/s of the last two of three launches of about 0.1 s, and the clock that rate
    implies (256 CUs x 4 SIMDs x 1024 FLOP per clock)."""
    import ctypes
    import torch
    path = os.path.join(ROOT, "paper_2507_21433_amd", "librc_probe.so")
    if not os.path.exists(path):
        raise RuntimeError("librc_probe.so is not built: run python -m paper_2507_21433_amd.build")
    lib = ctypes.CDLL(path)
    lib.rc_probe_mfma_f16.restype = ctypes.c_int
    lib.rc_probe_mfma_f16.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p]
    dev = "cuda:0"
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    gen = torch.Generator(device=dev)
    gen.manual_seed(4242)
    operands = torch.randn(16384, generator=gen, device=dev).to(torch.float16).contiguous()   # 32 KiB
    sink = torch.empty(cus * 256, dtype=torch.float32, device=dev)
    iters = 300000
    stream = torch.cuda.current_stream().cuda_stream
    rates = []
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        err = lib.rc_probe_mfma_f16(operands.data_ptr(), iters, sink.data_ptr(), cus, stream)
        if err:
            raise RuntimeError(f"rc_probe_mfma_f16: hipError {err}")
        e1.record()
        torch.cuda.synchronize()
        rates.append(cus * 4 * iters * 16 * 32768.0 / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    tflops = (rates[1] + rates[2]) / 2
    return {"pure_mfma_tflops": tflops, "implied_clock_ghz": tflops * 1e12 / (cus * 4 * 1024) / 1e9,
            "what": "back-to-back v_mfma_f32_32x32x16_f16, random operands, 4 waves per CU, no memory traffic; "
                    "three launches of 0.1 s, mean of the last two"}


def remap_sweep(args):
    """rc_remap_block_table on the table shape of cfg4 (64 tables of 776 entries per layer, 1024 new blocks, 50 176
    block ids) at growing layer counts, beside a device-to-device copy of the same number of bytes in the same run:
    the read-plus-write rate this chip reaches with nothing else to do."""
    import numpy as np
    import torch
    from paper_2507_21433_amd import binding as rc
    from paper_2507_21433_amd import synth
    dev = "cuda:0"
    w = synth.WORKLOADS[4]
    plan = synth.make_plan(w)
    rng = np.random.RandomState(99)
    live_ids = np.flatnonzero(plan.live)
    sweep = []
    for L in (64, 1024, 4096):
        tables = torch.as_tensor(plan.tables, device=dev)[None].repeat(L, 1, 1).contiguous()
        refcount = torch.as_tensor(plan.refcount, device=dev)[None].repeat(L, 1).contiguous()
        m = np.where(rng.rand(L, w.Q) < 0.4, live_ids[rng.randint(0, live_ids.size, size=(L, w.Q))], -1).astype(np.int32)
        match = torch.as_tensor(m, device=dev)
        qids = torch.as_tensor(plan.query_ids, device=dev)
        ws = torch.empty(rc.rc_remap_workspace_size(L, w.R, w.E, w.Q, w.NB), dtype=torch.uint8, device=dev)
        out = dict(tables=torch.empty_like(tables), refcount=torch.empty_like(refcount),
                   freed=torch.empty((L, w.Q), dtype=torch.uint8, device=dev),
                   n_remapped=torch.empty((L,), dtype=torch.int32, device=dev))
        ms = timed(torch, lambda: rc.rc_remap_block_table(tables, qids, None, match, w.P, w.NB, refcount, workspace=ws, out=out),
                   max(args.steps, 10))
        nbytes = L * (2 * w.R * w.E * 4 + 2 * w.NB * 4)           # tables and reference counts, each read once and written once
        src = torch.empty(nbytes // 2, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        copy_ms = timed(torch, lambda: dst.copy_(src), max(args.steps, 10))
        sweep.append({"layers": L, "bytes": nbytes, "ms": ms, "gb_per_s": nbytes / (ms * 1e-3) / 1e9,
                      "hbm_frac": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                      "copy_same_bytes_ms": copy_ms, "copy_gb_per_s": nbytes / (copy_ms * 1e-3) / 1e9,
                      "frac_of_copy": copy_ms / ms, "remapped_entries": int(out["n_remapped"].sum().item())})
        del tables, refcount, match, ws, out, src, dst
        torch.cuda.empty_cache()
    return sweep


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", type=int, default=4,
                    help="1..5: the workload of the headline (default 4, the largest that fits one GPU)")
    ap.add_argument("--configs", default="1,2,3,5",
                    help="workloads timed the same way before the headline and reported in `configs` ('none' = only the headline)")
    ap.add_argument("--step-only", type=int, default=0,
                    help="1 = the timed step of the headline workload and nothing else (the shape profiler runs use)")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (experiments only)")
    ap.add_argument("--cpu-pairs", type=float, default=1.2e7,
                    help="block pairs the CPU oracle is timed on for the headline (it scores about 0.85e6 per second on 16 "
                         "threads; 0 = skip); every other workload gets a third of it")
    ap.add_argument("--layer-mean", type=int, default=1, help="also time the layer-mean distance entry point (0 = skip)")
    ap.add_argument("--pat-samples", type=int, default=1 << 22, help="warm-up sample size for the percentile threshold (0 = skip)")
    ap.add_argument("--admit", type=int, default=1, help="also time the admission of unmatched blocks into the pool (0 = skip)")
    ap.add_argument("--streaming", type=int, default=4, help="consecutive decoding steps of the steady-state loop (0 = skip)")
    ap.add_argument("--candidates", type=int, default=16,
                    help="C of the candidate-restricted scoring timed beside the step (0 = skip)")
    ap.add_argument("--remap-sweep", type=int, default=1, help="also time the remap at 64 / 1024 / 4096 layers (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2507_21433_amd import binding as rc
    from paper_2507_21433_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    rc.lib()   # fail loudly if the HIP library is not built
    dev = "cuda:0"
    traffic, traffic_note = load_traffic()

    # a plain device-to-device copy of known size: the yardstick that scales the profiler's
    # FETCH_SIZE / WRITE_SIZE counters into bytes
    cal_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst
    torch.cuda.empty_cache()

    def workload(n):
        w = synth.WORKLOADS[n]
        return synth.scaled(w, L=args.layers) if args.layers else w

    configs = {}
    others = [] if (args.step_only or args.configs.strip().lower() in ("", "none")) else \
        [int(x) for x in args.configs.split(",") if int(x) != args.workload]
    side_errors = {}

    def guarded(what, fn):
        """A side measurement that fails must not take the headline with it: its error goes into the JSON line."""
        try:
            return fn()
        except Exception as e:   # noqa: BLE001
            log(f"{what} failed: {e!r}")
            side_errors[what] = repr(e)
            torch.cuda.empty_cache()
            return None

    for n in others:
        b = guarded(f"workload {n}", lambda: run_config(args, workload(n), traffic, extras=False, cpu_budget=args.cpu_pairs / 3))
        if b is not None:
            configs[b["config"]["workload"]] = b
    head = run_config(args, workload(args.workload), traffic, extras=not args.step_only,
                      cpu_budget=0 if args.step_only else args.cpu_pairs)
    if args.remap_sweep and not args.step_only:
        sweep = guarded("remap sweep", lambda: remap_sweep(args))
        if sweep is not None:
            head["kernels"]["rc_remap_block_table"]["sweep"] = sweep
    if not args.step_only:
        ceiling = guarded("pure-MFMA probe", mfma_probe)
        for b in (list(configs.values()) + [head]) if ceiling else []:
            r = b["roofline"]
            r["ceiling"] = dict(ceiling, frac_of_ceiling=r["tflops"] / ceiling["pure_mfma_tflops"])
    brief = {k: head[k] for k in ("value", "unit", "ms_per_step", "dtype", "config", "kv_gb_per_s", "roofline", "cpu_baseline")}
    brief["kernels"] = {k: v for k, v in head["kernels"].items() if "not in the step" not in k or "cold fill" in k}
    configs[head["config"]["workload"]] = brief
    configs = {k: configs[k] for k in sorted(configs)}

    line = {
        "metric": "block_pair_scores_per_s", "value": head["value"], "unit": "pairs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": head["config"],
        "kv_gb_per_s": head["kv_gb_per_s"],
        "roofline": head["roofline"],
        "cpu_baseline": head["cpu_baseline"],
        "kernels": head["kernels"],
        "streaming": head.get("streaming"),
        "matched_queries": head["matched_queries"], "remapped_entries": head["remapped_entries"],
        "configs": configs,
    }
    if traffic_note:
        line["traffic_note"] = traffic_note
    if side_errors or head.get("side_errors"):
        line["side_errors"] = dict(side_errors, **head.get("side_errors", {}))
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
