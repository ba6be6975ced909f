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

With --predictor the study covers the macro level of Section 2.3 instead: the popularity
persists over the micro-batches, the library keeps a routing history, derives a new
expert -> rank map from it and the same metrics are reported with and without that map.

    python -m paper_2604_19654_amd.straggler --ep 2 4 8 --dyn 2 4 8 --batches 8
    python -m paper_2604_19654_amd.straggler --predictor --ep 2 4 8 --batches 6 --warm 4
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
    """max - mean over the ranks (Section 3.1 Metrics), by the library."""
    return B.feplb_straggler(values)


def plan_counts(P: int, owner, counts, dyn_flag, dyn: int, tau: int = 0):
    """Per-rank token loads before and after the whole-expert plan, and the plan's moves."""
    slots = np.full(P, dyn, dtype=np.int32)
    moves, before, after, _ = B.feplb_plan(P, owner, counts, dyn_flag, slots, tau, B.PLAN_WHOLE)
    return moves, before, after


def placement(P: int, owner, counts, moves) -> List[List[int]]:
    """Row counts of the groups every rank runs, in expert order, with the plan's moves applied
    by the library.  Experts without rows form no group."""
    home = B.feplb_apply_moves(P, owner, moves)
    groups: List[List[int]] = [[] for _ in range(P)]
    for e in range(len(owner)):
        if counts[e] > 0:
            groups[int(home[e])].append(int(counts[e]))
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
          tau_list: Sequence[int] = (), keep_records: bool = False) -> Dict:
    """Mean token straggler before / after the plan for every dyn in dyn_list, and (for
    dyn = gemm_dyn) the mean GEMM straggler before / after, over n_batches micro-batches."""
    T = P * tokens_per_rank
    tok = {"before": [], **{f"dyn{n}": [] for n in dyn_list}}
    by_tau = {int(t): [] for t in tau_list}        # token straggler after the plan, dyn = gemm_dyn
    gemm = {"before": [], "after": []}
    layer = {"fwd_before": [], "bwd_before": [], "fwd_after": [], "bwd_after": []}
    records = []                                   # per micro-batch: what the figures were computed from
    timer = None
    for b in range(n_batches):
        # token rows are not needed: the smallest legal widths keep the generator cheap
        wl = workloads.make("C4", device=device, seed=seed0 + b, P=P, T=T, d=8, f=8, E=E, k=k)
        _ids, _w, counts_dev = B.feplb_route_topk(wl.logits, k)
        torch.cuda.synchronize()
        counts = counts_dev.cpu().numpy().astype(np.int64)
        owner = wl.owner()
        rec = {"seed": seed0 + b, "counts": counts, "loads": {}, "token_straggler": {}}
        records.append(rec)
        for t in by_tau:
            by_tau[t].append(straggler(plan_counts(P, owner, counts, wl.dyn_flags(gemm_dyn), gemm_dyn, t)[2]))
        first = True
        for n in dyn_list:
            moves, before, after = plan_counts(P, owner, counts, wl.dyn_flags(n), n, tau)
            if first:
                tok["before"].append(straggler(before))
                rec["loads"]["before"], rec["token_straggler"]["before"] = before, tok["before"][-1]
                first = False
            tok[f"dyn{n}"].append(straggler(after))
            rec["loads"][f"dyn{n}"], rec["token_straggler"][f"dyn{n}"] = after, tok[f"dyn{n}"][-1]
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
    if keep_records:
        out["records"] = records
    return out


def predictor_study(P: int, dyn: int, n_batches: int, warm: int, shift: int = 2, tokens_per_rank: int = 16384,
                    E: int = 128, k: int = 8, d: int = 6144, f: int = 2048, tau: int = 0, seed0: int = 7000,
                    device="cuda:0", with_gemm: bool = True, keep_records: bool = False, drift: int = 0,
                    replace_every: int = 0) -> Dict:
    """Macro level of Section 2.3 on synthetic routing whose popularity persists over the micro-batches
    of a run (one popularity seed, new logit noise per batch).  The first `warm` batches only feed the
    library's routing history; then the library derives a new expert -> rank map from it
    (feplb_place) and marks each rank's `dyn` busiest experts as dynamic (feplb_mark_dynamic).  On the
    remaining batches the token straggler (and, from the per-rank FFN times, the GEMM straggler) is
    reported for four set-ups: the contiguous map, the contiguous map with the per-micro-batch plan,
    the placed map, the placed map with the plan.  With drift > 0 that many random pairs of experts
    exchange their popularity between one micro-batch and the next, so the history lags behind;
    with replace_every > 0 the map is derived anew from the history after every so many measured
    micro-batches (the paper's "periodically"), starting from the map then in use.
    Sequencing only: routing, history, placement, plan and FFN are library calls."""
    if not 0 < warm < n_batches:
        raise B.FeplbError("predictor_study needs at least one micro-batch for the history and one to measure")
    T = P * tokens_per_rank
    per = E // P
    hist = np.zeros(E, dtype=np.int64)
    owner0 = None
    placed = None
    keys = ("contiguous", "contiguous+plan", "placed", "placed+plan")
    tok = {key: [] for key in keys}
    gemm = {key: [] for key in keys}
    records = []
    timer = None
    slots = np.full(P, dyn, dtype=np.int32)
    for b in range(n_batches):
        wl = workloads.make("C4", device=device, seed=seed0 + b, pop_seed=seed0, drift_swaps=b * drift, P=P, T=T, d=8, f=8,
                            E=E, k=k)
        _ids, _w, counts_dev = B.feplb_route_topk(wl.logits, k)
        torch.cuda.synchronize()
        counts = counts_dev.cpu().numpy().astype(np.int64)
        if owner0 is None:
            owner0 = wl.owner()
        if b < warm:
            B.feplb_history_update(hist, counts, shift if b else 0)     # the first batch starts the history
            continue
        if placed is None:
            owner1, load_before, load_after, migrated = B.feplb_place(P, hist, per, owner0)
            placed = dict(owner=owner1, predicted_before=load_before, predicted_after=load_after, migrated=migrated,
                          hist=hist.copy(), placements=[(b, migrated)])
        rec = {"seed": seed0 + b, "counts": counts, "loads": {}, "token_straggler": {}}
        records.append(rec)
        for name, owner in (("contiguous", owner0), ("placed", placed["owner"])):
            flags = B.feplb_mark_dynamic(P, owner, hist, dyn)
            moves, before, after, _ = B.feplb_plan(P, owner, counts, flags, slots, tau, B.PLAN_WHOLE)
            for key, loads, mv in ((name, before, []), (name + "+plan", after, moves)):
                tok[key].append(straggler(loads))
                rec["loads"][key], rec["token_straggler"][key] = loads, tok[key][-1]
                if with_gemm:
                    if timer is None:
                        timer = FfnTimer(d, f, max_rows=int(counts.sum()), max_groups=min(E, B.MAX_GROUPS), device=device)
                    gemm[key].append(straggler([timer.time_ms(s) for s in placement(P, owner, counts, mv)]))
        B.feplb_history_update(hist, counts, shift)
        if replace_every > 0 and (b - warm + 1) % replace_every == 0 and b + 1 < n_batches:
            owner1, _lb, _la, migrated = B.feplb_place(P, hist, per, placed["owner"])
            placed["owner"] = owner1
            placed["migrated"] += migrated
            placed["placements"].append((b + 1, migrated))
    out = {"P": P, "dyn": dyn, "batches": n_batches, "warm": warm, "shift": shift, "drift": drift, "replace_every": replace_every,
           "tokens_per_rank": tokens_per_rank,
           "E": E, "k": k, "migrated_experts": placed["migrated"],
           "predicted_max_load_rows": {"contiguous": float(placed["predicted_before"].max()) / (1 << B.HIST_FRAC_BITS),
                                       "placed": float(placed["predicted_after"].max()) / (1 << B.HIST_FRAC_BITS)},
           "token_straggler": {key: float(np.mean(v)) for key, v in tok.items()}}
    if with_gemm:
        out["gemm_straggler_ms"] = {key: float(np.mean(v)) for key, v in gemm.items()}
    if keep_records:
        out["records"] = records
        out["placed"] = placed
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
    ap.add_argument("--predictor", action="store_true",
                    help="macro level: routing whose popularity persists over the micro-batches; history -> placement, "
                         "then the four set-ups (contiguous / placed map, without / with the per-micro-batch plan)")
    ap.add_argument("--warm", type=int, default=4, help="micro-batches that only feed the history (--predictor)")
    ap.add_argument("--replace-every", type=int, default=0,
                    help="derive the map anew from the history after every so many measured micro-batches (--predictor; 0: once)")
    ap.add_argument("--drift", type=int, default=0,
                    help="pairs of experts that exchange their popularity between one micro-batch and the next (--predictor)")
    a = ap.parse_args()
    B.lib()
    if a.predictor:
        rows = []
        for P in a.ep:
            r = predictor_study(P, 4, a.batches + a.warm, a.warm, tokens_per_rank=a.tokens_per_rank, d=a.d, f=a.f, tau=a.tau,
                                with_gemm=not a.no_gemm, drift=a.drift, replace_every=a.replace_every)
            rows.append(r)
            print(json.dumps(r), flush=True)
        print("\n| EP | experts migrated | token straggler: contiguous | + plan | placed | placed + plan | GEMM straggler (ms): contiguous | + plan | placed | placed + plan |")
        print("|---|---|---|---|---|---|---|---|---|---|")
        for r in rows:
            t, g = r["token_straggler"], r.get("gemm_straggler_ms")
            keys = ("contiguous", "contiguous+plan", "placed", "placed+plan")
            print(f"| {r['P']} | {r['migrated_experts']} | " + " | ".join(f"{t[key]:.0f}" for key in keys) + " | " +
                  " | ".join(f"{g[key]:.3f}" if g else "-" for key in keys) + " |")
        return
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
