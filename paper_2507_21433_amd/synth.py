"""Seeded synthetic inputs for the reusable-KV-block search.

This module only draws inputs (random KV blocks, planted near-duplicates, block
tables with their reference counts).  It holds none of the method's arithmetic
and is the one module that the HIP path's tests and the CPU oracle's tests both
use.  Shapes follow QwQ-32B's KV cache (64 layers, 8 KV heads x 128, fp16,
16-token blocks, ~12.4k tokens per request); the share of planted near-duplicates
follows the 15-40 % step redundancy the paper reports (Sec. III).

The *plan* of a workload (which query slot copies which pool block, which pool
blocks are dead, the block tables) depends on the seed only and is drawn with
numpy on the host, so it is the same on every device.  The *values* are drawn
per layer with a torch generator on the requested device and rounded to
fp16 / bf16; a checker reads back the exact bytes it wants to check.
"""
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    L: int
    P: int
    Q: int
    T: int = 16
    H: int = 8
    Dh: int = 128
    dtype: str = "f16"          # "f16" | "bf16"
    mode: int = 0               # 0 = block score, 1 = per-head-all
    tau: float = 0.95
    seed: int = 0
    recipe: str = "planted"     # "planted" | "clustered"
    planted_frac: float = 0.0   # share of query slots that are noisy copies of pool blocks
    sigma: float = 0.1          # noise of a planted copy
    n_centroids: int = 0        # clustered recipe
    sigma_lo: float = 0.05
    sigma_hi: float = 0.5
    head_subset_noise: bool = False   # noise only on a random non-empty subset of heads
    tables: str = "generic"     # "generic" | "requests" | "single"
    R: int = 0
    E: int = 0
    dead_per_request: int = 0

    @property
    def D(self):
        return self.T * self.H * self.Dh

    @property
    def NB(self):
        return self.P + self.Q

    @property
    def torch_dtype(self):
        return torch.float16 if self.dtype == "f16" else torch.bfloat16

    @property
    def block_bytes(self):
        return 2 * self.D * 2   # one K plus one V tensor


# The five workloads of the benchmark definition.
WORKLOADS = {
    1: Workload("cfg1_tiny", L=1, P=256, Q=32, seed=0, planted_frac=8 / 32, sigma=0.1, tau=0.95,
                tables="single", R=1, E=40),
    2: Workload("cfg2_qwq32b_step", L=64, P=4096, Q=256, seed=1, planted_frac=0.30, sigma=0.15, tau=0.95,
                R=16, E=272),
    3: Workload("cfg3_clustered", L=64, P=16384, Q=1024, dtype="bf16", seed=2, recipe="clustered",
                n_centroids=128, tau=0.9, R=64, E=272),
    4: Workload("cfg4_high_concurrency", L=64, P=49152, Q=1024, seed=3, planted_frac=0.40, sigma=0.1, tau=0.95,
                tables="requests", R=64, E=776, dead_per_request=8),
    5: Workload("cfg5_small_model", L=32, P=8192, Q=512, T=32, mode=1, seed=4, planted_frac=0.20, sigma=0.1,
                tau=0.95, head_subset_noise=True, R=32, E=272),
}


def scaled(w: Workload, **kw) -> Workload:
    """Copy of a workload with some fields replaced (used for reduced-size test cases)."""
    d = {f: getattr(w, f) for f in w.__dataclass_fields__}
    d.update(kw)
    return Workload(**d)


@dataclass
class Plan:
    """Layer-independent structure of a workload."""
    planted_slots: np.ndarray     # [n_planted] query slots holding noisy copies
    planted_targets: np.ndarray   # [n_planted] pool block each one copies
    head_mask: Optional[np.ndarray]  # [n_planted][H] bool, heads that receive noise (None = all)
    live: np.ndarray              # [P] uint8
    tables: np.ndarray            # [R][E] int32, -1 = padding
    query_ids: np.ndarray         # [Q] int32 physical ids
    refcount: np.ndarray          # [NB] int32 = number of references in the tables


def make_plan(w: Workload) -> Plan:
    rng = np.random.RandomState(w.seed)
    P, Q = w.P, w.Q
    live = np.ones(P, dtype=np.uint8)
    query_ids = (P + np.arange(Q)).astype(np.int32)

    if w.tables == "requests":
        # Each request owns P/R consecutive pool blocks; the last `dead_per_request` of them were
        # released (dead) and are not in its table.  Its Q/R new blocks close the table.
        per, qper = P // w.R, Q // w.R
        assert per * w.R == P and qper * w.R == Q and w.E == per - w.dead_per_request + qper
        tables = np.empty((w.R, w.E), dtype=np.int32)
        for r in range(w.R):
            kept = np.arange(r * per, r * per + per - w.dead_per_request)
            live[r * per + per - w.dead_per_request:(r + 1) * per] = 0
            tables[r] = np.concatenate([kept, P + r * qper + np.arange(qper)])
    elif w.tables == "single":
        tables = np.full((1, w.E), -1, dtype=np.int32)
        tables[0, :Q] = query_ids
    else:
        per, qper = P // w.R, Q // w.R
        assert qper >= 1 and w.E >= per + qper
        tables = np.full((w.R, w.E), -1, dtype=np.int32)
        for r in range(w.R):
            tables[r, :per] = r * per + np.arange(per)
            tables[r, per:per + qper] = P + r * qper + np.arange(qper)

    n_planted = int(round(w.planted_frac * Q)) if w.recipe == "planted" else 0
    slots = np.sort(rng.choice(Q, size=n_planted, replace=False)).astype(np.int64)
    live_ids, dead_ids = np.flatnonzero(live), np.flatnonzero(live == 0)
    n_dead_t = min(n_planted // 8, dead_ids.size)   # plants aimed at dead blocks must not match
    tg = np.concatenate([rng.choice(dead_ids, size=n_dead_t, replace=False) if n_dead_t else np.empty(0, np.int64),
                         rng.choice(live_ids, size=n_planted - n_dead_t, replace=False)])
    targets = tg[rng.permutation(n_planted)].astype(np.int64) if n_planted else tg.astype(np.int64)
    head_mask = None
    if w.head_subset_noise and n_planted:
        head_mask = rng.rand(n_planted, w.H) < 0.5
        empty = ~head_mask.any(axis=1)
        head_mask[empty, rng.randint(0, w.H, size=int(empty.sum()))] = True

    refcount = np.bincount(tables[tables >= 0].ravel(), minlength=w.NB).astype(np.int32)
    return Plan(slots, targets, head_mask, live, tables, query_ids, refcount)


def _randn(shape, g, device):
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


def make_layer(w: Workload, plan: Plan, layer: int, device="cpu"):
    """KV blocks of one layer: dict(kq, vq [Q][T][H][Dh], kp, vp [P][T][H][Dh]) in the workload's dtype."""
    g = torch.Generator(device=device)
    g.manual_seed(int(w.seed) * 1_000_003 + int(layer) * 7919 + 17)
    dt, D = w.torch_dtype, w.D
    out = {}
    if w.recipe == "clustered":
        cent = {n: _randn((w.n_centroids, D), g, device) for n in ("k", "v")}
        for side, n in (("p", w.P), ("q", w.Q)):
            cid = torch.randint(0, w.n_centroids, (n,), generator=g, device=device)
            sig = w.sigma_lo + (w.sigma_hi - w.sigma_lo) * torch.rand((n, 1), generator=g, device=device)
            for kv in ("k", "v"):
                out[kv + side] = (cent[kv][cid] + sig * _randn((n, D), g, device)).to(dt)
    else:
        for kv in ("k", "v"):
            out[kv + "p"] = _randn((w.P, D), g, device).to(dt)
            out[kv + "q"] = _randn((w.Q, D), g, device).to(dt)
        if plan.planted_slots.size:
            slots = torch.as_tensor(plan.planted_slots, device=device)
            tg = torch.as_tensor(plan.planted_targets, device=device)
            for kv in ("k", "v"):
                noise = w.sigma * _randn((slots.numel(), D), g, device)
                if plan.head_mask is not None:
                    hm = torch.as_tensor(plan.head_mask, device=device, dtype=torch.float32)
                    noise = (noise.view(-1, w.T, w.H, w.Dh) * hm[:, None, :, None]).reshape(-1, D)
                out[kv + "q"][slots] = (out[kv + "p"][tg].float() + noise).to(dt)
    return {n: t.view(-1, w.T, w.H, w.Dh) for n, t in out.items()}


def make_problem(w: Workload, device="cpu", layers=None):
    """All (or the listed) layers stacked: tensors [L'][n][T][H][Dh] plus the plan's arrays as tensors."""
    plan = make_plan(w)
    layers = list(range(w.L)) if layers is None else list(layers)
    dt = w.torch_dtype
    kv = {n: torch.empty((len(layers), cnt, w.T, w.H, w.Dh), dtype=dt, device=device)
          for n, cnt in (("kq", w.Q), ("vq", w.Q), ("kp", w.P), ("vp", w.P))}
    for i, l in enumerate(layers):
        lay = make_layer(w, plan, l, device)
        for n in kv:
            kv[n][i].copy_(lay[n])
        del lay
    nl = len(layers)
    kv["live"] = torch.as_tensor(plan.live, device=device)[None].repeat(nl, 1).contiguous()
    kv["tables"] = torch.as_tensor(plan.tables, device=device)[None].repeat(nl, 1, 1).contiguous()
    kv["refcount"] = torch.as_tensor(plan.refcount, device=device)[None].repeat(nl, 1).contiguous()
    kv["query_ids"] = torch.as_tensor(plan.query_ids, device=device)
    kv["plan"] = plan
    kv["layers"] = layers
    return kv


def bits(t: torch.Tensor) -> np.ndarray:
    """Raw 16-bit patterns of an fp16 / bf16 tensor as a numpy uint16 array (host copy)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
