"""Buffers and call sequence of one training step of the grouped expert FFN (forward that keeps
the SwiGLU derivatives, then the backward pass; paper Section 3.2 reports both times).  Only
allocation and sequencing live here: every step is a library call."""
from __future__ import annotations

from typing import Dict, Sequence

import torch

from . import binding as B


class FfnTrainingStep:
    """Holds what feplb_grouped_ffn (training form) and feplb_grouped_ffn_backward need for G
    groups and up to R_cap permuted rows: H, the SwiGLU derivatives p|q (turned into da|db by the
    backward), Yp, dXp,
    the fp32 weight gradients, the transposed-weight scratch and the workspace."""

    def __init__(self, R_cap: int, G: int, d: int, f: int, device="cuda:0", dxp_dtype=torch.float32):
        dev = torch.device(device)
        self.R_cap, self.G, self.d, self.f = max(R_cap, 32), G, d, f
        R = self.R_cap
        self.H = torch.empty((R, f), dtype=torch.bfloat16, device=dev)
        self.AB = torch.empty((R, 2 * f), dtype=torch.bfloat16, device=dev)
        self.Yp = torch.empty((R, d), dtype=torch.float32, device=dev)
        self.dXp = torch.empty((R, d), dtype=dxp_dtype, device=dev)
        self.dW_gate = [torch.empty((d, f), dtype=torch.float32, device=dev) for _ in range(G)]
        self.dW_up = [torch.empty((d, f), dtype=torch.float32, device=dev) for _ in range(G)]
        self.dW_down = [torch.empty((f, d), dtype=torch.float32, device=dev) for _ in range(G)]
        self.WT = torch.empty((max(B.feplb_grouped_ffn_backward_wt_bytes(G, d, f), 16),), dtype=torch.uint8, device=dev)
        self.ws = torch.empty((B.feplb_grouped_ffn_workspace_bytes(R, G),), dtype=torch.uint8, device=dev)

    def _need_rows(self, t, name):
        # the kernels size their grids by R_cap and the weight gradients read whole 32-row windows
        if t.shape[0] < self.R_cap or t.shape[1] != self.d:
            raise B.FeplbError(f"{name} must be [{self.R_cap}, {self.d}] (rows past the last group are not used), "
                               f"got {tuple(t.shape)}")

    def forward(self, Xp, offsets, w_gate, w_up, w_down, stream=None):
        """Xp bf16 [R_cap,d] (a materialised permuted copy, which the backward reads again)."""
        self._need_rows(Xp, "Xp")
        B.feplb_grouped_ffn(Xp, offsets, 0, self.G, self.d, self.f, w_gate, w_up, w_down, self.H, self.Yp,
                            ws=self.ws, stream=stream, AB=self.AB)
        return self.Yp

    def backward(self, Xp, offsets, w_gate, w_up, w_down, dYp, phases=B.BWD_ALL, stream=None):
        """dYp bf16 [R_cap,d] -> dXp; the weight gradients land in dW_gate / dW_up / dW_down."""
        self._need_rows(Xp, "Xp")
        self._need_rows(dYp, "dYp")
        B.feplb_grouped_ffn_backward(Xp, offsets, 0, self.G, self.d, self.f, w_gate, w_up, w_down, self.H, self.AB,
                                     dYp, self.dXp, self.dW_gate, self.dW_up, self.dW_down, WT=self.WT,
                                     phases=phases, ws=self.ws, stream=stream)
        return self.dXp


def setup_from_prepared(p, seed: int = 4242, dxp_dtype=torch.float32):
    """Training-step inputs on a workload that runner.step has already run once: the permuted copy
    Xp of the step's own token rows (feplb_permute), its offsets, the groups' weights, a seeded
    synthetic upstream gradient dYp ~ N(0,1) in bf16, and the buffers.
    Returns (step, Xp, offsets, (w_gate, w_up, w_down), dYp)."""
    from . import runner
    lay, b, wl = p.layer, p.layer.buf, p.wl
    G = len(p.groups)
    dev = wl.X.device
    W = runner.group_weights(p)
    weights = tuple([w[i] for w in W] for i in range(3))
    R_cap = max(lay.R_cap, 32)
    Xp = torch.zeros((R_cap, lay.d), dtype=torch.bfloat16, device=dev)
    offsets = b.offsets[: G + 1]
    B.feplb_permute(b.topk_ids, lay.E, p.groups, wl.X, lay.R_cap, Xp, offsets, b.row_src, b.inv, b.ws_permute)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    dYp = torch.empty((R_cap, lay.d), dtype=torch.float32, device=dev).normal_(generator=gen).to(torch.bfloat16)
    return FfnTrainingStep(R_cap, G, lay.d, lay.f, device=dev, dxp_dtype=dxp_dtype), Xp, offsets, weights, dYp


class LayerBackward:
    """The layer's backward pass behind a training forward on the same buffers (FfnTrainingStep.forward
    on the permuted copy, then the combine): dY [T,d] -> dYp (combine backward, which also yields the
    routing weights' gradient) -> dXp and the weight gradients (FFN backward) -> dX (row gather backward:
    the combine with unit weights) and dlogits (router backward).  Sequencing and buffers only."""

    def __init__(self, T: int, E: int, k: int, step: FfnTrainingStep):
        dev = step.H.device
        self.T, self.E, self.k, self.step = T, E, k, step
        self.dYp = torch.empty((step.R_cap, step.d), dtype=torch.bfloat16, device=dev)
        self.dw = torch.empty((T, k), dtype=torch.float32, device=dev)
        self.ones = torch.ones((T, k), dtype=torch.float32, device=dev)
        self.dX = torch.empty((T, step.d), dtype=torch.bfloat16, device=dev)
        self.dlogits = torch.empty((T, E), dtype=torch.float32, device=dev)

    def run(self, dY, Xp, offsets, weights, topk_ids, topk_w, inv, events=None):
        """events: optional dict that receives HipEvents recorded between the steps."""
        st = self.step
        wg, wu, wd = weights

        def mark(name):
            if events is not None:
                events.setdefault(name, B.HipEvent()).record(None)
        mark("start")
        B.feplb_combine_backward(dY, st.Yp, inv, topk_w, self.T, self.k, st.d, self.dYp, self.dw)
        mark("combine_backward")
        st.backward(Xp, offsets, wg, wu, wd, self.dYp)
        mark("ffn_backward")
        B.feplb_unpermute_combine(st.dXp, inv, self.ones, self.T, self.k, st.d, Y=self.dX)
        mark("gather_backward")
        B.feplb_route_topk_backward(topk_ids, topk_w, self.dw, self.E, self.dlogits)
        mark("route_backward")
        return self.dX, self.dlogits


def time_phases(step: FfnTrainingStep, Xp, offsets, w_gate, w_up, w_down, dYp, reps: int = 5) -> Dict[str, float]:
    """Milliseconds per call (HIP events on the default stream) of the training forward and of each
    backward phase on its own, and of the whole backward in one call."""
    e0, e1 = B.HipEvent(), B.HipEvent()

    def timed(fn):
        fn()
        e0.record(None)
        for _ in range(reps):
            fn()
        e1.record(None)
        e1.synchronize()
        return e0.elapsed_ms(e1) / reps

    out = {"forward_keeping_derivatives": timed(lambda: step.forward(Xp, offsets, w_gate, w_up, w_down))}
    step.forward(Xp, offsets, w_gate, w_up, w_down)
    step.backward(Xp, offsets, w_gate, w_up, w_down, dYp)      # leaves tile table and transposes in place
    for name, ph in (("transpose", B.BWD_TRANSPOSE), ("dgrad", B.BWD_DGRAD), ("wgrad", B.BWD_WGRAD),
                     ("wgrad_accumulating", B.BWD_WGRAD | B.BWD_ACCUMULATE), ("backward", B.BWD_ALL)):
        out[name] = timed(lambda ph=ph: step.backward(Xp, offsets, w_gate, w_up, w_down, dYp, phases=ph))
    return out
