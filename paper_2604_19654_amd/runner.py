"""Sets a named synthetic workload up on the GPU and runs layer steps on it.
Used by the benchmark, the smoke check and the GPU tests so that all three
launch the library in the same configuration.  No arithmetic of the method
lives here: sizing comes from the library's own routing counts and plan.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch

import workloads
from . import binding as B
from .layer import RankLayer


@dataclass
class Prepared:
    wl: workloads.Workload
    layer: RankLayer
    rebalanced: bool
    groups: List[Tuple[int, int, int]]           # static layer: the group table
    weights: List[Tuple]                         # static layer: per-group (Wg, Wu, Wd)
    rank: int
    R: int                                       # rows this rank runs
    counts: np.ndarray                           # per-expert assignment counts (from the library's router)
    # rebalanced layer
    dyn_flag: Optional[np.ndarray] = None
    slots: Optional[np.ndarray] = None
    static_weights: Optional[Dict[int, Tuple]] = None
    remote_sources: Optional[Dict[int, torch.Tensor]] = None
    moves: Optional[list] = None
    source_kind: str = "device"


def _route_counts(wl) -> np.ndarray:
    _, _, counts = B.feplb_route_topk(wl.logits, wl.k)
    torch.cuda.synchronize()
    return counts.cpu().numpy().astype(np.int64)


def prepare(name: str, device="cuda:0", yp_dtype=torch.float32, source_kind="device", fused_gather=True,
            r_cap: Optional[int] = None, **override) -> Prepared:
    """yp_dtype: type of the expert outputs between the down GEMM and the combine: fp32 (default)
    or bf16, which is faster (half the bytes through the down epilogue and the combine) but adds a
    rounding per expert output.
    fused_gather: the gate/up GEMM gathers the token rows itself (no permuted copy of X).
    source_kind: where the replicas' weights are copied from -- "device"
    (a second buffer in HBM, standing in for a peer GPU's memory) or "pinned"
    (page-locked host memory).
    r_cap: rows the layer's buffers hold.  Default: exactly the rows of this batch, which is
    right as long as the same logits are stepped; a caller that feeds other batches through the
    same layer passes a bound (T*k always suffices) and may ask `layer.rows_overflow()`."""
    wl = workloads.make(name, device=device, **override)
    counts = _route_counts(wl)
    if wl.n_dyn == 0:
        experts = [int(e) for e in wl.local_experts()]
        groups = [(e, 0, B.ORD_MAX) for e in experts]
        R = int(counts[experts].sum())
        weights = [wl.expert_weights(e) for e in experts]
        layer = RankLayer(wl.T, wl.E, wl.k, wl.d, wl.f, R_cap=r_cap or max(R, 1), G_cap=len(groups), device=device,
                          yp_dtype=yp_dtype, fused_gather=fused_gather)
        return Prepared(wl, layer, False, groups, weights, wl.rank, R, counts)
    # rebalanced share: the library's plan picks the receiving rank and the replicas
    dyn_flag = wl.dyn_flags(4)
    slots = np.full(wl.P, wl.n_dyn, dtype=np.int32)
    moves, before, after, rank = B.feplb_plan(wl.P, wl.owner(), counts, dyn_flag, slots, 0, B.PLAN_OVERFLOW,
                                              wl.rank)
    static = [int(e) for e in wl.local_experts(rank)]
    R = int(counts[static].sum() + sum(m[3] for m in moves))
    static_weights = {e: wl.expert_weights(e) for e in static}
    remote = {}
    for (e, *_r) in moves:
        flat = torch.cat([m.reshape(-1) for m in wl.expert_weights(e)])
        if source_kind == "pinned":
            host = torch.empty(flat.shape, dtype=flat.dtype, pin_memory=True)
            host.copy_(flat)
            flat = host
        remote[int(e)] = flat
    layer = RankLayer(wl.T, wl.E, wl.k, wl.d, wl.f, R_cap=r_cap or max(R, 1), G_cap=len(static) + wl.n_dyn,
                      device=device, yp_dtype=yp_dtype, n_slots=wl.n_dyn, fused_gather=fused_gather)
    groups = [(e, 0, B.ORD_MAX) for e in static] + [(m[0], m[4], m[4] + m[3]) for m in moves]
    return Prepared(wl, layer, True, groups, [], rank, R, counts, dyn_flag, slots, static_weights, remote,
                    moves, source_kind)


def step(p: Prepared, mark=False, overlap=True, early_static=True):
    """One pass of the whole hot path over the workload's batch. Returns Y (bf16 [T,d]).
    Rebalanced share: by default the timeline of Section 2.3 -- the static experts' permute and
    FFN are launched before the host has the plan, the replicas' groups are appended behind the
    static FFN (needs overlap).  early_static=False plans first and permutes all groups at once."""
    wl = p.wl
    if not p.rebalanced:
        return p.layer.forward(wl.logits, wl.X, p.groups, p.weights, mark=mark)
    if early_static and overlap:
        Y, info = p.layer.forward_rebalanced_early_static(wl.logits, wl.X, wl.P, wl.owner(), p.dyn_flag, p.slots,
                                                          p.rank, p.static_weights, p.remote_sources, mark=mark)
    else:
        Y, info = p.layer.forward_rebalanced(wl.logits, wl.X, wl.P, wl.owner(), p.dyn_flag, p.slots, p.rank,
                                             p.static_weights, p.remote_sources, mark=mark, overlap=overlap)
    p.moves = info["moves"]
    p.groups = info["groups"]
    return Y


def group_weights(p: Prepared):
    """Per-group (Wg, Wu, Wd) tensors as the layer used them (replicas read from the staging slots)."""
    if not p.rebalanced:
        return list(p.weights)
    ns = len(p.static_weights)
    static = [g[0] for g in p.groups[:ns]]
    return [p.static_weights[e] for e in static] + [p.layer.slot_views(i) for i in range(len(p.groups) - ns)]
