"""One EP rank's MoE layer as a sequence of library calls (paper Section 2.3,
per-micro-batch timeline): route -> [counts to host -> plan -> stage dynamic
experts' weights on a side stream] -> permute -> static experts' FFN ->
wait for the staging event -> dynamic experts' FFN -> combine.

By default the permute step computes the row indices only and the gate/up GEMM
gathers the token rows while loading them (fused_gather); with fused_gather=False
the permute step writes the permuted copy Xp and the GEMM reads that.

Only sequencing, buffer ownership and stream plumbing live here; every step is
a call into libfeplb.so.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import binding as B


@dataclass
class LayerBuffers:
    topk_ids: torch.Tensor
    topk_w: torch.Tensor
    counts: torch.Tensor
    counts_host: torch.Tensor
    offsets: torch.Tensor
    row_src: torch.Tensor
    inv: torch.Tensor
    Xp: Optional[torch.Tensor]
    H: torch.Tensor
    Yp: torch.Tensor
    Y: torch.Tensor
    ws_permute: torch.Tensor
    ws_ffn: torch.Tensor
    slots: Optional[torch.Tensor]


class RankLayer:
    """Pre-allocates every buffer once (sized by R_cap rows and G_cap groups) so
    that a step launches kernels only."""

    def __init__(self, T, E, k, d, f, R_cap, G_cap, device="cuda", yp_dtype=torch.float32, n_slots=0,
                 fused_gather=True):
        self.T, self.E, self.k, self.d, self.f = T, E, k, d, f
        self.fused_gather = fused_gather
        self.R_cap, self.G_cap, self.n_slots = R_cap, G_cap, n_slots
        dev = torch.device(device)
        i32 = dict(dtype=torch.int32, device=dev)
        bf = dict(dtype=torch.bfloat16, device=dev)
        self.expert_elems = 3 * d * f
        self.buf = LayerBuffers(
            topk_ids=torch.empty((T, k), **i32),
            topk_w=torch.empty((T, k), dtype=torch.float32, device=dev),
            counts=torch.empty((E,), **i32),
            counts_host=torch.empty((E,), dtype=torch.int32, pin_memory=True),
            offsets=torch.zeros((G_cap + 1,), **i32),
            row_src=torch.empty((max(R_cap, 1),), **i32),
            inv=torch.empty((max(T * k, 1),), **i32),
            Xp=None if fused_gather else torch.empty((R_cap, d), **bf),
            H=torch.empty((R_cap, f), **bf),
            Yp=torch.empty((R_cap, d), dtype=yp_dtype, device=dev),
            Y=torch.empty((T, d), **bf),
            ws_permute=torch.empty((B.feplb_permute_workspace_bytes(T, k, E, G_cap),), dtype=torch.uint8, device=dev),
            ws_ffn=torch.empty((B.feplb_grouped_ffn_workspace_bytes(R_cap, G_cap),), dtype=torch.uint8, device=dev),
            slots=torch.empty((n_slots, self.expert_elems), **bf) if n_slots else None,
        )
        self.side_stream = torch.cuda.Stream(device=dev) if n_slots else None      # staging copies
        self.append_stream = torch.cuda.Stream(device=dev) if n_slots else None    # late permute of the replicas
        self.staged = B.HipEvent() if n_slots else None
        self.appended = B.HipEvent() if n_slots else None
        self.timeline: Dict[str, B.HipEvent] = {}

    # -- helpers ---------------------------------------------------------
    def rows_overflow(self, G: int) -> int:
        """Rows of the last permutation over G groups beyond the layer's capacity (0: all fit).
        Reads offsets[G] back, so it synchronises; rows past the capacity are neither computed
        nor combined (their slots count as not local), which is safe but drops work."""
        return max(0, int(self.buf.offsets[G].item()) - self.R_cap)

    def _mark(self, name: str, on: bool):
        if on:
            ev = self.timeline.get(name)
            if ev is None:
                ev = self.timeline[name] = B.HipEvent()
            ev.record(None)

    def slot_views(self, i: int):
        d, f = self.d, self.f
        s = self.buf.slots[i]
        return s[: d * f].view(d, f), s[d * f: 2 * d * f].view(d, f), s[2 * d * f:].view(f, d)

    def _permute(self, groups, X, first=0, stream=None):
        """Groups first .. first+len(groups)-1 of the layer's group table.  first > 0 appends to an
        earlier call (rows continue at offsets[first])."""
        b = self.buf
        G = len(groups)
        off = b.offsets[first: first + G + 1]
        Xin, Xp = (None, None) if self.fused_gather else (X, b.Xp)   # fused: indices only
        B.feplb_permute(b.topk_ids, self.E, groups, Xin, self.R_cap, Xp, off, b.row_src, b.inv, b.ws_permute,
                        stream=stream, append=first > 0)

    def _ffn_range(self, X, g0, g1, wg, wu, wd, tag, mark):
        """One ragged launch per GEMM for groups [g0, g1).  With mark=True the
        schedule / gate_up / down launches are issued by separate calls so that
        HIP events can bracket each GEMM kernel on its stream."""
        b = self.buf
        src = (X, b.row_src) if self.fused_gather else (b.Xp, None)
        args = (src[0], b.offsets, g0, g1, self.d, self.f, wg, wu, wd, b.H, b.Yp)
        kw = dict(ws=b.ws_ffn, row_src=src[1], k=self.k)
        if not mark:
            B.feplb_grouped_ffn(*args, phases=B.FFN_ALL, **kw)
            return
        B.feplb_grouped_ffn(*args, phases=B.FFN_SCHEDULE, **kw)
        self._mark(tag + "_scheduled", True)
        B.feplb_grouped_ffn(*args, phases=B.FFN_GATE_UP, **kw)
        self._mark(tag + "_gate_up", True)
        B.feplb_grouped_ffn(*args, phases=B.FFN_DOWN, **kw)
        self._mark(tag + "_down", True)

    # -- static-only layer (no dynamic experts) ---------------------------
    def forward(self, logits, X, groups: Sequence[Tuple[int, int, int]], weights: Sequence[Tuple], mark=False):
        """groups[g] = (expert, ord_lo, ord_hi); weights[g] = (W_gate, W_up, W_down). Returns Y."""
        b = self.buf
        G = len(groups)
        self._mark("start", mark)
        B.feplb_route_topk(logits, self.k, b.topk_ids, b.topk_w, b.counts)
        self._mark("routed", mark)
        self._permute(groups, X)
        self._mark("permuted", mark)
        wg, wu, wd = ([w[i] for w in weights] for i in range(3))
        self._ffn_range(X, 0, G, wg, wu, wd, "static", mark)
        B.feplb_unpermute_combine(b.Yp, b.inv, b.topk_w, self.T, self.k, self.d, b.Y)
        self._mark("combined", mark)
        return b.Y

    def capture_forward(self, logits, X, groups: Sequence[Tuple[int, int, int]], weights: Sequence[Tuple]):
        """Records one `forward` on these very buffers into a HIP graph and returns it; `replay()`
        then re-runs the step (router to combine, about ten launches) as one submission, which is
        what the small workloads need: their step is as long as its launch gaps.  The step has no
        host round trip and the library launches nothing but kernels (no memset nodes).  The
        graph reads `logits`, `X` and the weights where they are now and writes `self.buf.Y`."""
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.forward(logits, X, groups, weights, mark=False)
        return g

    # -- rebalanced layer: static experts + replicas of the hottest foreign experts
    def forward_rebalanced_early_static(self, logits, X, P, owner, dyn_flag, slots, this_rank,
                                        static_weights: Dict[int, Tuple],
                                        remote_sources: Dict[int, torch.Tensor], mark=False):
        """Section 2.3 timeline in full: the static experts (this rank's own, known without the
        plan) are permuted and their FFN is launched right after the router; the host meanwhile
        reads the counts back on the side stream, plans, stages the replicas' weights and appends
        the replicas' groups to the permutation, all behind the static FFN.  `this_rank` must be
        the rank the plan will pick (the caller knows its own rank).  Returns (Y, info)."""
        b = self.buf
        main, side = torch.cuda.current_stream(), self.side_stream
        if side is None or this_rank < 0:
            raise B.FeplbError("early static launch needs staging slots and a known rank")
        per = self.E // P
        static = list(range(this_rank * per, (this_rank + 1) * per))
        Gs = len(static)
        self._mark("start", mark)
        B.feplb_route_topk(logits, self.k, b.topk_ids, b.topk_w, b.counts)
        self._mark("routed", mark)
        routed = self.timeline.setdefault("_routed", B.HipEvent())
        routed.record(main)
        # static range: needs nothing from the host
        self._permute([(e, 0, B.ORD_MAX) for e in static], X)
        self._mark("permuted", mark)
        permuted = self.timeline.setdefault("_permuted", B.HipEvent())
        permuted.record(main)
        wstat = [static_weights[e] for e in static]
        slots_w = [self.slot_views(i) for i in range(self.n_slots)]
        wg, wu, wd = ([w[i] for w in wstat + slots_w] for i in range(3))
        self._ffn_range(X, 0, Gs, wg, wu, wd, "static", mark)
        # meanwhile: counts to the host on the side stream (waits for the router only), plan
        B.feplb_stream_wait(side, routed)
        with torch.cuda.stream(side):
            b.counts_host.copy_(b.counts, non_blocking=True)
        side.synchronize()
        n = b.counts_host.numpy().astype(np.int64)
        moves, before, after, rank = B.feplb_plan(P, owner, n, dyn_flag, slots, 0, B.PLAN_OVERFLOW, this_rank)
        if rank != this_rank:
            raise B.FeplbError("the plan picked another receiving rank than the one given")
        if len(moves) > self.n_slots:
            raise B.FeplbError("more replicas than staging slots")
        groups = [(e, 0, B.ORD_MAX) for e in static] + [(e, lo, lo + rows) for (e, _src, _dst, rows, lo) in moves]
        G = len(groups)
        # replicas: weights by the copy engine on the side stream, their rows appended to the
        # permutation, both behind the static FFN (the append shares the permute workspace and
        # buffers with the static call, hence the wait for it)
        if moves:
            if mark:
                self.timeline.setdefault("copy_start", B.HipEvent()).record(side)
            for i, (e, *_rest) in enumerate(moves):
                B.feplb_stage_weights(b.slots[i], remote_sources[e], side, None)
            self.staged.record(side)
            if mark:
                self.timeline.setdefault("copy_end", B.HipEvent()).record(side)
            # the append on a stream of its own: its small kernels wait for compute units the
            # static GEMM holds, and the copies must not queue behind them
            aux = self.append_stream
            B.feplb_stream_wait(aux, permuted)
            self._permute(groups[Gs:], X, first=Gs, stream=aux)
            self.appended.record(aux)
            B.feplb_stream_wait(main, self.staged)
            B.feplb_stream_wait(main, self.appended)
            self._mark("staged", mark)
            self._ffn_range(X, Gs, G, wg, wu, wd, "dynamic", mark)
        self._mark("dynamic_done", mark)
        B.feplb_unpermute_combine(b.Yp, b.inv, b.topk_w, self.T, self.k, self.d, b.Y)
        self._mark("combined", mark)
        info = dict(rank=rank, moves=moves, groups=groups, load_before=before, load_after=after, n=n)
        return b.Y, info

    def forward_rebalanced(self, logits, X, P, owner, dyn_flag, slots, this_rank,
                           static_weights: Dict[int, Tuple], remote_sources: Dict[int, torch.Tensor],
                           mark=False, overlap=True):
        """The rank runs its own experts as the static range and `slots[this_rank]`
        replicas as the dynamic range.  remote_sources[e] is one contiguous bf16
        tensor [gate | up | down] of expert e living where the copy engine reads it
        (another device buffer or pinned host memory).  Returns (Y, info)."""
        b = self.buf
        main = torch.cuda.current_stream()
        self._mark("start", mark)
        B.feplb_route_topk(logits, self.k, b.topk_ids, b.topk_w, b.counts)
        self._mark("routed", mark)
        # per-expert counts to the host: the plan is CPU work triggered by the router (Section 2.3)
        b.counts_host.copy_(b.counts, non_blocking=True)
        main.synchronize()
        n = b.counts_host.numpy().astype(np.int64)
        moves, before, after, rank = B.feplb_plan(P, owner, n, dyn_flag, slots, 0, B.PLAN_OVERFLOW, this_rank)
        per = self.E // P
        static = list(range(rank * per, (rank + 1) * per))
        groups = [(e, 0, B.ORD_MAX) for e in static]
        groups += [(e, lo, lo + rows) for (e, _src, _dst, rows, lo) in moves]
        Gs, G = len(static), len(static) + len(moves)
        if len(moves) > self.n_slots:
            raise B.FeplbError("more replicas than staging slots")
        # the permute kernels go first: the GPU has been idle since the router finished
        self._permute(groups, X)
        self._mark("permuted", mark)
        # weights of the replicas: copy engine, side stream, off the compute units.  The side
        # stream waits for what is queued on the main stream (the previous step's readers of the
        # slots; the few permute kernels above ride along).
        side = self.side_stream if overlap else main
        if overlap:
            side.wait_stream(main)
        if mark and moves:
            self.timeline.setdefault("copy_start", B.HipEvent()).record(side)
        for i, (e, *_rest) in enumerate(moves):
            last = i == len(moves) - 1
            B.feplb_stage_weights(b.slots[i], remote_sources[e], side, self.staged if last else None)
        if mark and moves:
            self.timeline.setdefault("copy_end", B.HipEvent()).record(side)
        wlist = [static_weights[e] for e in static] + [self.slot_views(i) for i in range(len(moves))]
        wg, wu, wd = ([w[i] for w in wlist] for i in range(3))
        self._ffn_range(X, 0, Gs, wg, wu, wd, "static", mark)
        if moves:
            B.feplb_stream_wait(main, self.staged)
            self._mark("staged", mark)
            self._ffn_range(X, Gs, G, wg, wu, wd, "dynamic", mark)
        self._mark("dynamic_done", mark)
        B.feplb_unpermute_combine(b.Yp, b.inv, b.topk_w, self.T, self.k, self.d, b.Y)
        self._mark("combined", mark)
        info = dict(rank=rank, moves=moves, groups=groups, load_before=before, load_after=after, n=n)
        return b.Y, info
