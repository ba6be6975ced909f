"""Straggler study on synthetic routing (paper Section 3.1 "Metrics"; Section 3.3,
token and GEMM straggler tables; Section 3.5, sweep over the dynamic expert count).

For P simulated EP ranks the study routes a micro-batch with the library's router,
asks the library's host plan (whole-expert mode, Section 2.3) where the dynamic
experts should run, and reports the two metrics the paper defines:

  token straggler = max over ranks of the token count, minus the mean;
  GEMM straggler  = max over ranks of the grouped-FFN time, minus the mean.

The per-rank FFN times come from running every rank's share of groups one after the
other on the one GPU through feplb_grouped_ffn, once with the static placement and
once with the plan's placement.  Only sequencing lives here; routing, plan and FFN
are library calls.  Inputs are synthetic (Zipf-biased logits, one popularity
permutation per micro-batch): the paper's traces are not public, so the figures show
the mechanism, not the paper's numbers.

    python -m paper_2604_19654_amd.straggler --ep 2 4 8 --dyn 2 4 8 --batches 8
"""
from __future__ import annotations

import argparse
import json
from typing import Dict, List, Sequence

import numpy as np
import torch

import workloads

from . import binding as B


def straggler(values) -> float:
    """max - mean (Section 3.1 Metrics)."""
    v = np.asarray(values, dtype=np.float64)
    return float(v.max() - v.mean())


def plan_counts(P: int, owner, counts, dyn_flag, dyn: int, tau: int = 0):
    """Per-rank token loads before and after the whole-expert plan, and the plan's moves."""
    slots = np.full(P, dyn, dtype=np.int32)
    moves, before, after, _ = B.feplb_plan(P, owner, counts, dyn_flag, slots, tau, B.PLAN_WHOLE)
    return moves, before, after


def placement(P: int, owner, counts, moves) -> List[List[int]]:
    """Row counts of the groups every rank runs: its own experts that stay, then the experts
    it receives.  Experts without rows form no group."""
    home = {int(e): int(owner[e]) for e in range(len(owner))}
    for (e, _src, dst, _rows, _lo) in moves:
        home[int(e)] = int(dst)
    groups: List[List[int]] = [[] for _ in range(P)]
    for e in range(len(owner)):
        if counts[e] > 0:
            groups[home[e]].append(int(counts[e]))
    return groups


class FfnTimer:
    """Times feplb_grouped_ffn for lists of group sizes; buffers sized once for `max_rows`."""

    def __init__(self, d: int, f: int, max_rows: int, max_groups: int, device="cuda:0", seed=7):
        dev = torch.device(device)
        g = torch.Generator(device=dev)
        g.manual_seed(seed)
        self.d, self.f, self.max_rows, self.max_groups = d, f, max_rows, max_groups
        self.Xp = torch.empty((max_rows, d), dtype=torch.float32, device=dev).normal_(generator=g).to(torch.bfloat16)
        self.H = torch.empty((max_rows, f), dtype=torch.bfloat16, device=dev)
        self.Yp = torch.empty((max_rows, d), dtype=torch.float32, device=dev)
        self.ws = torch.empty((B.feplb_grouped_ffn_workspace_bytes(max_rows, max_groups),), dtype=torch.uint8, device=dev)
        # distinct weights per group slot: time does not depend on the values, but sharing one
        # matrix between groups would flatter the caches
        def w(shape):
            return (torch.empty(shape, dtype=torch.float32, device=dev).normal_(generator=g) * 0.02).to(torch.bfloat16)
        self.wg = [w((d, f)) for _ in range(max_groups)]
        self.wu = [w((d, f)) for _ in range(max_groups)]
        self.wd = [w((f, d)) for _ in range(max_groups)]
        self.e0, self.e1 = B.HipEvent(), B.HipEvent()

    def time_train_ms(self, sizes: Sequence[int], reps: int = 2):
        """(forward keeping the SwiGLU derivatives, backward) of one share, in ms."""
        from .training import FfnTrainingStep
        G = len(sizes)
        if G == 0 or sum(sizes) == 0:
            return 0.0, 0.0
        if G > self.max_groups or sum(sizes) > self.max_rows:
            raise B.FeplbError("FfnTimer: share larger than the buffers")
        if getattr(self, "_train", None) is None or self._train.G != G:
            self._train = None       # buffers of the previous group count go first
            self._train = FfnTrainingStep(self.max_rows, G, self.d, self.f, device=self.Xp.device)
            self._dYp = self.Xp.flip(0)
        st = self._train
        off = torch.tensor(np.concatenate([[0], np.cumsum(sizes)]), dtype=torch.int32, device=self.Xp.device)
        w = (self.wg[:G], self.wu[:G], self.wd[:G])
        out = []
        for fn in (lambda: st.forward(self.Xp, off, *w), lambda: st.backward(self.Xp, off, *w, self._dYp)):
            fn()
            self.e0.record(None)
            for _ in range(reps):
                fn()
            self.e1.record(None)
            self.e1.synchronize()
            out.append(self.e0.elapsed_ms(self.e1) / reps)
        return out[0], out[1]

    def time_ms(self, sizes: Sequence[int], reps: int = 3) -> float:
        G = len(sizes)
        if G == 0 or sum(sizes) == 0:
            return 0.0
        if G > self.max_groups or sum(sizes) > self.max_rows:
            raise B.FeplbError("FfnTimer: share larger than the buffers")
        off = torch.tensor(np.concatenate([[0], np.cumsum(sizes)]), dtype=torch.int32, device=self.Xp.device)
        args = (self.Xp, off, 0, G, self.d, self.f, self.wg[:G], self.wu[:G], self.wd[:G], self.H, self.Yp)
        B.feplb_grouped_ffn(*args, ws=self.ws)   # warm-up
        self.e0.record(None)
        for _ in range(reps):
            B.feplb_grouped_ffn(*args, ws=self.ws)
        self.e1.record(None)
        self.e1.synchronize()
        return self.e0.elapsed_ms(self.e1) / reps


def study(P: int, dyn_list: Sequence[int], n_batches: int, tokens_per_rank: int = 16384, E: int = 128,
          k: int = 8, d: int = 6144, f: int = 2048, tau: int = 0, seed0: int = 5000, gemm_dyn: int = 4,
          device="cuda:0", with_gemm: bool = True, with_backward: bool = False,
          tau_list: Sequence[int] = ()) -> Dict:
    """Mean token straggler before / after the plan for every dyn in dyn_list, and (for
    dyn = gemm_dyn) the mean GEMM straggler before / after, over n_batches micro-batches."""
    T = P * tokens_per_rank
    tok = {"before": [], **{f"dyn{n}": [] for n in dyn_list}}
    by_tau = {int(t): [] for t in tau_list}        # token straggler after the plan, dyn = gemm_dyn
    gemm = {"before": [], "after": []}
    layer = {"fwd_before": [], "bwd_before": [], "fwd_after": [], "bwd_after": []}
    timer = None
    for b in range(n_batches):
        # token rows are not needed: the smallest legal widths keep the generator cheap
        wl = workloads.make("C4", device=device, seed=seed0 + b, P=P, T=T, d=8, f=8, E=E, k=k)
        _ids, _w, counts_dev = B.feplb_route_topk(wl.logits, k)
        torch.cuda.synchronize()
        counts = counts_dev.cpu().numpy().astype(np.int64)
        owner = wl.owner()
        for t in by_tau:
            by_tau[t].append(straggler(plan_counts(P, owner, counts, wl.dyn_flags(gemm_dyn), gemm_dyn, t)[2]))
        first = True
        for n in dyn_list:
            moves, before, after = plan_counts(P, owner, counts, wl.dyn_flags(n), n, tau)
            if first:
                tok["before"].append(straggler(before))
                first = False
            tok[f"dyn{n}"].append(straggler(after))
            if with_gemm and n == gemm_dyn:
                shares_before = placement(P, owner, counts, [])
                shares_after = placement(P, owner, counts, moves)
                if timer is None:
                    timer = FfnTimer(d, f, max_rows=int(counts.sum()), max_groups=min(E, B.MAX_GROUPS), device=device)
                gemm["before"].append(straggler([timer.time_ms(s) for s in shares_before]))
                gemm["after"].append(straggler([timer.time_ms(s) for s in shares_after]))
                if with_backward:
                    # the layer waits for its slowest rank (Section 3.2): max over the ranks' times
                    for key, shares in (("before", shares_before), ("after", shares_after)):
                        times = [timer.time_train_ms(s) for s in shares]
                        layer["fwd_" + key].append(max(t[0] for t in times))
                        layer["bwd_" + key].append(max(t[1] for t in times))
    out = {"P": P, "batches": n_batches, "tokens_per_rank": tokens_per_rank, "E": E, "k": k, "tau": tau,
           "token_straggler": {key: float(np.mean(v)) for key, v in tok.items()}}
    base = out["token_straggler"]["before"]
    out["token_reduction_pct"] = {key: 100.0 * (1.0 - v / base) for key, v in out["token_straggler"].items() if key != "before"}
    if by_tau:
        out["token_straggler_by_tau"] = {str(t): float(np.mean(v)) for t, v in by_tau.items()}
    if with_gemm and gemm["before"]:
        gb, ga = float(np.mean(gemm["before"])), float(np.mean(gemm["after"]))
        out["gemm_straggler_ms"] = {"before": gb, f"dyn{gemm_dyn}": ga, "d": d, "f": f}
        out["gemm_reduction_pct"] = 100.0 * (1.0 - ga / gb) if gb > 0 else 0.0
    if layer["fwd_before"]:
        out["slowest_rank_ffn_ms"] = {key: float(np.mean(v)) for key, v in layer.items()}
    return out


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--ep", type=int, nargs="+", default=[2, 4, 8])
    ap.add_argument("--dyn", type=int, nargs="+", default=[2, 4, 8])
    ap.add_argument("--batches", type=int, default=8)
    ap.add_argument("--tokens-per-rank", type=int, default=16384)
    ap.add_argument("--d", type=int, default=6144)
    ap.add_argument("--f", type=int, default=2048)
    ap.add_argument("--tau", type=int, default=0)
    ap.add_argument("--tau-sweep", type=int, nargs="*", default=[],
                    help="thresholds tau (minimum rows for an expert to be moved) to sweep at dyn=4")
    ap.add_argument("--no-gemm", action="store_true")
    ap.add_argument("--backward", action="store_true",
                    help="also time every rank's FFN training step (forward keeping the SwiGLU derivatives, backward) and report the slowest rank's times before and after the plan")
    a = ap.parse_args()
    B.lib()
    rows = []
    for P in a.ep:
        r = study(P, a.dyn, a.batches, a.tokens_per_rank, d=a.d, f=a.f, tau=a.tau, with_gemm=not a.no_gemm, with_backward=a.backward,
                  tau_list=a.tau_sweep)
        rows.append(r)
        print(json.dumps(r), flush=True)
    print("\n| EP | token straggler before | " + " | ".join(f"dyn={n}" for n in a.dyn) + " | GEMM straggler before (ms) | dyn=4 (ms) |")
    print("|---|---|" + "---|" * len(a.dyn) + "---|---|")
    for r in rows:
        t = r["token_straggler"]
        cells = [f"{t[f'dyn{n}']:.0f} (-{r['token_reduction_pct'][f'dyn{n}']:.0f}%)" for n in a.dyn]
        g = r.get("gemm_straggler_ms")
        gcells = [f"{g['before']:.3f}", f"{g['dyn4']:.3f} (-{r['gemm_reduction_pct']:.0f}%)"] if g and "dyn4" in g else ["-", "-"]
        print(f"| {r['P']} | {t['before']:.0f} | " + " | ".join(cells) + " | " + " | ".join(gcells) + " |")
    if a.backward:
        print("\n| EP | slowest rank's FFN forward / backward before (ms) | after, dyn=4 (ms) |")
        print("|---|---|---|")
        for r in rows:
            m = r.get("slowest_rank_ffn_ms")
            if m:
                print(f"| {r['P']} | {m['fwd_before']:.2f} / {m['bwd_before']:.2f} | {m['fwd_after']:.2f} / {m['bwd_after']:.2f} |")
    if a.tau_sweep:
        print("\n| EP | before | " + " | ".join(f"tau={t}" for t in a.tau_sweep) + " |")
        print("|---|---|" + "---|" * len(a.tau_sweep))
        for r in rows:
            bt = r["token_straggler_by_tau"]
            base = r["token_straggler"]["before"]
            print(f"| {r['P']} | {base:.0f} | " + " | ".join(f"{bt[str(t)]:.0f} (-{100 * (1 - bt[str(t)] / base):.0f}%)" for t in a.tau_sweep) + " |")


if __name__ == "__main__":
    main()
