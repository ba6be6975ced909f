#!/usr/bin/env python3
"""Benchmark of one EP rank's MoE hot path on one MI355X.

A step is one pass of the whole path (route -> [plan + staging] -> permute ->
grouped SwiGLU FFN -> combine) over one synthetic batch that is already
resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4] [--no-cpu-baseline] [--only]

value      = FFN flops of the step (6*d*f per permuted row) / wall time of the WHOLE step
roofline   = the gate/up GEMM (the dominant kernel): 4*d*f flops per row over its
             average launch duration, measured with HIP events on the launch stream
rooflines  = the same kind of object for the down GEMM, the combine, the permute step, the router
cpu_baseline = the CPU oracle timed on a bounded sample of the same workload, with the parity verdict
other_workloads = the four other workloads as short forward-only runs (skipped with --only)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 (no sparsity)
HBM_PEAK_GBPS = 8000.0           # MI355X HBM3E
# HBM bytes per launch (read, written) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled by what the
# same counters read for the row-copy and combine kernels of the same run (sizes known); see the named profile.
# The figures belong to the kernel source they were measured on: bench.py reports them only while
# csrc/ffn.hip still has that content (sha256), and null otherwise.
MEASURED_TRAFFIC = {
    "C4": {"profile": "profiles/hbm_traffic_C4_C3_pmc.md",
           "ffn_hip_sha256": "e220b4efd4c5d5adfadee6c4b4c8fb1beb505f7a128794e6795867ee6e9636ce",
           "gate_up": {"read": 2496533 * 1024 * 2.0, "written": 262140 * 1024},       # FETCH_SIZE KiB x 2.000, WRITE_SIZE KiB
           "down": {"read": 1271943 * 1024 * 2.0, "written": 1573573 * 1024}},
    "C3": {"profile": "profiles/hbm_traffic_C4_C3_pmc.md",
           "ffn_hip_sha256": "e220b4efd4c5d5adfadee6c4b4c8fb1beb505f7a128794e6795867ee6e9636ce",
           "gate_up": {"read": 454829 * 1024 * 2.0, "written": 61188 * 1024},
           "down": {"read": 227325 * 1024 * 2.0, "written": 326958 * 1024}},
}
METRIC = "grouped-FFN TFLOP/s & % bf16 MFMA peak per rank share; permute/combine GB/s"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_workload(name, steps, warmup, source_kind="device", fused_gather=True, yp_dtype="f32", early_static=True):
    import numpy as np
    import torch
    from paper_2604_19654_amd import runner

    p = runner.prepare(name, "cuda:0", source_kind=source_kind, fused_gather=fused_gather,
                       yp_dtype=torch.bfloat16 if yp_dtype == "bf16" else torch.float32)
    wl, layer = p.wl, p.layer
    for _ in range(warmup):
        runner.step(p, mark=True, early_static=early_static)
    torch.cuda.synchronize()
    # Every timed step records into an event set of its own, read after the last step has drained: the host
    # never waits between steps (a rebalanced step still waits, inside the step, for its counts read-back).
    # (The event sets are created here, before the clock starts: creating events inside the timed loop can
    # make the runtime grow its signal pool in the middle of a step.)
    from paper_2604_19654_amd import binding as B
    names = list(layer.timeline)
    timelines = [{n: B.HipEvent() for n in names} for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for tl in timelines:
        layer.timeline = tl
        runner.step(p, mark=True, early_static=early_static)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    acc = {}
    per_step = []
    for tl in timelines:
        def span(a, b, key):
            if a in tl and b in tl:
                acc[key] = acc.get(key, 0.0) + tl[a].elapsed_ms(tl[b])
        span("start", "routed", "route")
        span("start", "combined", "step_events")
        per_step.append(tl["start"].elapsed_ms(tl["combined"]))
        if p.rebalanced:
            span("static_scheduled", "static_gate_up", "gate_up")
            span("static_gate_up", "static_down", "down")
            span("dynamic_scheduled", "dynamic_gate_up", "gate_up")
            span("dynamic_gate_up", "dynamic_down", "down")
            span("copy_start", "copy_end", "copy")
            span("static_down", "staged", "wait_for_copy")
            span("dynamic_done", "combined", "combine")
            # plan first: counts read-back, host plan and the permute of all groups; early static
            # launch: the permute of the static groups only (the rest happens behind the static FFN)
            span("routed", "permuted", "permute_static" if early_static else "plan_stage_permute")
        else:
            span("routed", "permuted", "permute")
            span("static_scheduled", "static_gate_up", "gate_up")
            span("static_gate_up", "static_down", "down")
            span("static_down", "combined", "combine")
    acc.setdefault("copy", 0.0)
    ms = {k: v / steps for k, v in acc.items() if not k.startswith("_")}
    n_up = 2 if (p.rebalanced and len(p.groups) > len(p.static_weights)) else 1
    R, d, f, T, k = p.R, wl.d, wl.f, wl.T, wl.k
    ffn_flops = 6.0 * d * f * R
    yp_bytes = layer.buf.Yp.element_size()
    res = dict(
        workload=name, T=T, R=R, d=d, f=f, E=wl.E, k=k, groups=len(p.groups), rank=p.rank,
        ms_per_step=wall_ms, ms=ms,
        step_events_ms_median=float(np.median(per_step)), step_events_ms_min=float(np.min(per_step)),
        ffn_tflops_step=ffn_flops / (wall_ms * 1e-3) / 1e12,
        ffn_tflops_kernels=ffn_flops / ((ms["gate_up"] + ms["down"]) * 1e-3) / 1e12,
        gate_up_tflops=4.0 * d * f * R / (ms["gate_up"] * 1e-3) / 1e12,
        down_tflops=2.0 * d * f * R / (ms["down"] * 1e-3) / 1e12,
        gate_up_launches_per_step=n_up,
        gate_up_ms_per_launch=ms["gate_up"] / n_up,
        combine_gbps=(R * d * yp_bytes + T * d * 2 + T * k * 8) / (ms["combine"] * 1e-3) / 1e9,
        route_gbps=(T * wl.E * 4 + T * k * 8) / (ms["route"] * 1e-3) / 1e9,
    )
    if not p.rebalanced:
        # the same step recorded once into a HIP graph and replayed: one submission instead of
        # about ten launches (a share without replicas has no host round trip inside the step)
        graph = layer.capture_forward(wl.logits, wl.X, p.groups, p.weights)
        for _ in range(warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        res["graph_replay_ms_per_step"] = (time.perf_counter() - t0) * 1e3 / steps
        res["ffn_tflops_step_graph_replay"] = ffn_flops / (res["graph_replay_ms_per_step"] * 1e-3) / 1e12
        del graph
    # per-group rows as the device has them (read back once, after the timed region): the algorithmic
    # bytes of a launch count the weights of its NON-EMPTY groups only
    G = len(p.groups)
    offs = layer.buf.offsets[: G + 1].cpu().numpy().astype(np.int64)
    rows_g = np.diff(offs)
    ranges = [(0, len(p.static_weights)), (len(p.static_weights), G)] if n_up == 2 else [(0, G)]
    launches = []
    for (g0, g1) in ranges:
        r_l, ne = int(rows_g[g0:g1].sum()), int((rows_g[g0:g1] > 0).sum())
        launches.append({"groups": [g0, g1], "rows": r_l, "nonempty_groups": ne,
                         "gate_up_bytes": ne * 2 * d * f * 2 + r_l * d * 2 + r_l * f * 2,
                         "down_bytes": ne * d * f * 2 + r_l * f * 2 + r_l * d * yp_bytes})
    res["group_rows"] = rows_g.tolist()
    res["nonempty_groups"] = int((rows_g > 0).sum())
    res["launches"] = launches
    res["fused_gather"] = fused_gather
    res["yp_dtype"] = yp_dtype
    # the permute step with its row gather (X -> Xp), timed on its own when the step's GEMM gathers the rows itself
    res["permute_with_gather_ms"] = ms["permute"] if ("permute" in ms and not fused_gather) else _permute_ms(p, steps)
    res["permute_gbps"] = (2 * R * d * 2 + T * k * 8 + R * 4) / (res["permute_with_gather_ms"] * 1e-3) / 1e9
    # the row copy alone: the step with the gather minus the index kernels timed without it
    res["permute_indices_ms"] = _permute_ms(p, steps, with_rows=False)
    gather_ms = max(res["permute_with_gather_ms"] - res["permute_indices_ms"], 1e-6)
    res["hbm_kernels"] = {
        "peak_gbps": HBM_PEAK_GBPS,
        "combine": {"ms": ms["combine"], "gbps": res["combine_gbps"], "frac": res["combine_gbps"] / HBM_PEAK_GBPS},
        "permute_with_gather": {"ms": res["permute_with_gather_ms"], "gbps": res["permute_gbps"],
                                "frac": res["permute_gbps"] / HBM_PEAK_GBPS},
        "row_gather_alone": {"ms": gather_ms, "gbps": 2 * R * d * 2 / (gather_ms * 1e-3) / 1e9,
                             "frac": 2 * R * d * 2 / (gather_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS},
    }
    if p.rebalanced:
        nbytes = sum(t.numel() * t.element_size() for t in p.remote_sources.values())
        engine = ("blit kernel on the compute units (same-device copy: the stand-in for a peer GPU's memory; a peer copy over xGMI would use an SDMA engine)"
                  if p.source_kind == "device" else "SDMA engine, pinned host memory over PCIe")
        if early_static:
            # the copies run beside the static GEMM (and, from device memory, as a blit kernel that
            # competes with it for compute units), so this is a span, not a copy rate
            res["staging"] = dict(bytes=nbytes, source=p.source_kind, engine=engine, copy_span_ms=ms["copy"],
                                  wait_after_static_ms=ms["wait_for_copy"])
        else:
            res["staging"] = dict(bytes=nbytes, source=p.source_kind, engine=engine, copy_ms=ms["copy"],
                                  copy_gbps=nbytes / (ms["copy"] * 1e-3) / 1e9,
                                  wait_after_static_ms=ms["wait_for_copy"])
        res["moves"] = p.moves
        # the host plan's latency on this machine's CPU (Section 2.3 budgets about 50 us on one core): both modes on the
        # step's own counts, median of 200 calls through the C ABI
        from paper_2604_19654_amd import binding as B
        owner, flags = wl.owner(), wl.dyn_flags(4)
        lat = {}
        for mode_name, args in (("whole_expert_greedy", (64, B.PLAN_WHOLE, -1)), ("overflow_replicas", (0, B.PLAN_OVERFLOW, p.rank))):
            ts = []
            for _ in range(200):
                t1 = time.perf_counter()
                B.feplb_plan(wl.P, owner, p.counts, flags, p.slots, *args)
                ts.append(time.perf_counter() - t1)
            lat[mode_name] = float(np.median(ts)) * 1e6
        res["plan_latency_us"] = lat
    res["pct_mfma_peak_ffn_kernels"] = 100.0 * res["ffn_tflops_kernels"] / MFMA_BF16_PEAK_TFLOPS
    res["reference_copy_gbps"] = _reference_copy_gbps(layer.buf.Y)
    res["reference_dense_gemm"] = _reference_dense_gemm(R, d, f, wl.X.device)
    res["rooflines"] = _rooflines(name, res)
    return p, res


def _reference_copy_gbps(buf):
    """What a plain device-to-device copy of the same size reaches on this machine (torch's elementwise
    copy kernel, read + written bytes): the plateau of 1:1 read/write traffic, for context."""
    import torch
    from paper_2604_19654_amd import binding as B
    dst = torch.empty_like(buf)
    e0, e1 = B.HipEvent(), B.HipEvent()
    dst.copy_(buf)
    e0.record(None)
    for _ in range(10):
        dst.copy_(buf)
    e1.record(None)
    e1.synchronize()
    return 2 * buf.numel() * buf.element_size() / (e0.elapsed_ms(e1) / 10 * 1e-3) / 1e9


def _reference_dense_gemm(R, d, f, device):
    """Context only, never part of the path: what the vendor library's plain dense bf16 GEMM (torch.matmul) reaches
    on this machine for one matrix product of the gate/up GEMM's size, [R, d] x [d, 2f], and one of the down GEMM's
    size, [R, f] x [f, d] -- one group each, no ragged tiles, no row gather, no SwiGLU, bf16 output."""
    import torch
    from paper_2604_19654_amd import binding as B
    out = {"what": "torch.matmul, bf16 in and out, one dense product of each GEMM's size"}
    try:
        gen = torch.Generator(device=device)
        gen.manual_seed(99)
        for key, (m, kk, n) in (("gate_up", (R, d, 2 * f)), ("down", (R, f, d))):
            a = torch.empty((m, kk), dtype=torch.float32, device=device).normal_(generator=gen).to(torch.bfloat16)
            w = (torch.empty((kk, n), dtype=torch.float32, device=device).normal_(generator=gen) * 0.02).to(torch.bfloat16)
            c = torch.empty((m, n), dtype=torch.bfloat16, device=device)
            e0, e1 = B.HipEvent(), B.HipEvent()
            for _ in range(3):
                torch.matmul(a, w, out=c)
            e0.record(None)
            for _ in range(5):
                torch.matmul(a, w, out=c)
            e1.record(None)
            e1.synchronize()
            ms = e0.elapsed_ms(e1) / 5
            tf = 2.0 * m * kk * n / (ms * 1e-3) / 1e12
            out[key] = {"shape": [m, kk, n], "ms": ms, "tflops": tf, "frac_of_mfma_peak": tf / MFMA_BF16_PEAK_TFLOPS}
            del a, w, c
    except Exception as exc:      # a reference figure must never break the benchmark
        out["error"] = str(exc)
    return out


def _traffic(name, kernel):
    """Measured HBM bytes per launch of `kernel` on workload `name`, or None when there is no
    measurement for the kernel source as it stands."""
    import hashlib
    m = MEASURED_TRAFFIC.get(name)
    if not m or not m.get(kernel):
        return None
    src = os.path.join(ROOT, "paper_2604_19654_amd", "csrc", "ffn.hip")
    with open(src, "rb") as fh:
        if hashlib.sha256(fh.read()).hexdigest() != m["ffn_hip_sha256"]:
            return None
    return m[kernel]["read"] + m[kernel]["written"]


def _rooflines(name, res):
    """One roofline object per kernel of the step: algorithmic flops or bytes per launch (no padding, no empty
    groups) over the average launch duration measured with HIP events on the launch stream."""
    d, f, R, T, k, E = res["d"], res["f"], res["R"], res["T"], res["k"], res["E"]
    ms, n = res["ms"], res["gate_up_launches_per_step"]
    L = res["launches"]
    yp_bytes = 2 if res["yp_dtype"] == "bf16" else 4

    def mfma(kernel, key, flops_per_row, bytes_key):
        achieved = flops_per_row * R / (ms[key] * 1e-3) / 1e12
        return {"kernel": kernel, "bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": _traffic(name, key),
                "traffic_unit": "HBM bytes per launch, read + written (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE)",
                "traffic_profile": MEASURED_TRAFFIC.get(name, {}).get("profile"),
                "launches_per_step": n, "avg_launch_ms": ms[key] / n, "flops_per_launch": flops_per_row * R / n,
                "algorithmic_bytes_per_launch": sum(l[bytes_key] for l in L) / n,
                "per_launch": [{"rows": l["rows"], "nonempty_groups": l["nonempty_groups"], "algorithmic_bytes": l[bytes_key]} for l in L]}

    def hbm(kernel, t_ms, nbytes, traffic=None):
        achieved = nbytes / (t_ms * 1e-3) / 1e9
        return {"kernel": kernel, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "avg_launch_ms": t_ms, "algorithmic_bytes_per_launch": nbytes}

    out = {
        "gate_up": mfma("grouped_gemm_kernel<0,true,false> (gate/up GEMM + SwiGLU)", "gate_up", 4.0 * d * f, "gate_up_bytes"),
        "down": mfma("grouped_gemm_kernel<1,%s,false> (down GEMM)" % ("true" if yp_bytes == 2 else "false"), "down", 2.0 * d * f, "down_bytes"),
        "combine": hbm("combine_kernel", ms["combine"], R * d * yp_bytes + T * d * 2 + T * k * 8),
        "permute_with_gather": hbm("chunk_hist + chunk_scan + group_offsets + assign_rows + gather_rows_kernel",
                                   res["permute_with_gather_ms"], 2 * R * d * 2 + T * k * 8 + R * 4),
        "row_gather_alone": hbm("gather_rows_kernel (the step above minus its index kernels)",
                                res["hbm_kernels"]["row_gather_alone"]["ms"], 2 * R * d * 2),
        # the router is bound by its vector ALU work, not by the 67 MB it reads (T*E*4 + T*k*8 bytes): about 45 vector
        # operations per logit (5 per entry of the sorted list of k = 8, plus the exponentials and the histogram),
        # against 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3e12 lane operations per second
        "route": {"kernel": "route_topk kernel", "bound": "alu", "achieved": 45.0 * T * E / (ms["route"] * 1e-3) / 1e12,
                  "peak": 256 * 4 * 16 * 2.4e9 / 1e12, "unit": "T lane-op/s",
                  "frac": 45.0 * T * E / (ms["route"] * 1e-3) / (256 * 4 * 16 * 2.4e9), "traffic": None,
                  "avg_launch_ms": ms["route"], "hbm_gbps": res["route_gbps"], "hbm_frac": res["route_gbps"] / HBM_PEAK_GBPS},
    }
    return out


def _permute_ms(p, steps, with_rows=True):
    """feplb_permute on the step's own routing: with the row gather into a permuted copy, or the
    index part alone."""
    import torch
    from paper_2604_19654_amd import binding as B
    lay, b = p.layer, p.layer.buf
    G = len(p.groups)
    Xp = torch.empty((lay.R_cap, lay.d), dtype=torch.bfloat16, device=p.wl.X.device) if with_rows else None
    args = (b.topk_ids, lay.E, p.groups, p.wl.X if with_rows else None, lay.R_cap, Xp, b.offsets[: G + 1], b.row_src,
            b.inv, b.ws_permute)
    e0, e1 = B.HipEvent(), B.HipEvent()
    B.feplb_permute(*args)
    e0.record(None)
    for _ in range(steps):
        B.feplb_permute(*args)
    e1.record(None)
    e1.synchronize()
    return e0.elapsed_ms(e1) / steps


def training_leg(p, steps):
    """Forward (keeping the SwiGLU derivatives) and backward of the grouped FFN on the step's own
    groups and token rows, with a synthetic upstream gradient; reported beside the forward step,
    not part of `value`."""
    import torch
    from paper_2604_19654_amd.training import setup_from_prepared, time_phases, LayerBackward
    lay, b, wl = p.layer, p.layer.buf, p.wl
    st, Xp, offsets, (wg, wu, wd), dYp = setup_from_prepared(p)
    reps = max(3, min(steps, 10))
    ms = time_phases(st, Xp, offsets, wg, wu, wd, dYp, reps=reps)
    # the layer's whole backward chain behind that forward: combine, FFN, row gather, router
    gen = torch.Generator(device=wl.X.device)
    gen.manual_seed(4243)
    dY = torch.empty((wl.T, lay.d), dtype=torch.float32, device=wl.X.device).normal_(generator=gen).to(torch.bfloat16)
    lb = LayerBackward(wl.T, wl.E, wl.k, st)
    ev, chain = {}, {}
    st.forward(Xp, offsets, wg, wu, wd)
    lb.run(dY, Xp, offsets, (wg, wu, wd), b.topk_ids, b.topk_w, b.inv, events=ev)
    names = ["start", "combine_backward", "ffn_backward", "gather_backward", "route_backward"]
    for _ in range(reps):
        lb.run(dY, Xp, offsets, (wg, wu, wd), b.topk_ids, b.topk_w, b.inv, events=ev)
        ev["route_backward"].synchronize()
        for a_, b_ in zip(names[:-1], names[1:]):
            chain[b_] = chain.get(b_, 0.0) + ev[a_].elapsed_ms(ev[b_]) / reps
    chain["total"] = sum(chain.values())
    R, d, T, k = p.R, lay.d, wl.T, wl.k
    yp_bytes = st.Yp.element_size()
    fl = 2.0 * p.R * lay.d * lay.f
    return dict(ms=ms, layer_backward_ms=chain,
                combine_backward_gbps=(T * d * 2 + R * d * yp_bytes + R * d * 2 + T * k * 12) / (chain["combine_backward"] * 1e-3) / 1e9,
                gather_backward_gbps=(R * d * st.dXp.element_size() + T * d * 2 + T * k * 8) / (chain["gather_backward"] * 1e-3) / 1e9,
                flops_forward=3 * fl, flops_backward=6 * fl,
                forward_tflops=3 * fl / (ms["forward_keeping_derivatives"] * 1e-3) / 1e12,
                dgrad_tflops=3 * fl / (ms["dgrad"] * 1e-3) / 1e12,
                wgrad_tflops=3 * fl / (ms["wgrad"] * 1e-3) / 1e12,
                backward_tflops=6 * fl / (ms["backward"] * 1e-3) / 1e12,
                backward_over_forward=ms["backward"] / ms["forward_keeping_derivatives"],
                note="backward = weight transposes + dH GEMM with the SwiGLU derivative + dXp GEMM + three ragged "
                     "weight-gradient GEMMs (fp32 out); upstream gradient synthetic; Xp materialised")


def cpu_baseline(p, budget_tokens):
    """The oracle as it stands, on a bounded sample: full routing, plan and
    permutation (integer work), then the layer's per-token definition on a
    strided sample of tokens; the FFN flops of the sampled local rows over the
    time of that last part give the oracle's TFLOP/s."""
    import numpy as np
    import torch
    from oracle import feplb_oracle as orc
    from tests.util import f64, row_rel_err, ROW_TOL, layer_tokens_with_format_bound

    wl = p.wl
    t0 = time.perf_counter()
    ids, w, counts = orc.route_topk(wl.logits.cpu().numpy(), wl.k)
    if p.rebalanced:
        this = orc.pick_receiver(wl.P, wl.owner(), counts)
        moves, _, _ = orc.plan_overflow(wl.P, wl.owner(), counts, wl.dyn_flags(4), p.slots, this)
        groups = [(int(e), 0, orc.INT32_MAX) for e in wl.local_experts(this)] + \
                 [(m[0], m[4], m[4] + m[3]) for m in moves]
    else:
        groups = [(int(e), 0, orc.INT32_MAX) for e in wl.local_experts()]
    offsets, row_src, inv = orc.permute(ids, groups)
    t_int = time.perf_counter() - t0
    stride = max(1, wl.T // budget_tokens)
    toks = np.arange(0, wl.T, stride)
    keep = inv.reshape(wl.T, wl.k)[toks] >= 0
    rows = int(keep.sum())
    tt = torch.from_numpy(toks).to(wl.X.device)
    x = f64(wl.X[tt])
    weights_of = lambda e: tuple(f64(m) for m in wl.expert_weights(e))
    t1 = time.perf_counter()
    want = orc.moe_tokens(x, ids[toks], w[toks], keep, weights_of)
    t_ffn = time.perf_counter() - t1
    got = f64(p.layer.buf.Y[tt])
    row_err = row_rel_err(got, want)
    err = float(row_err.max())
    # the same measure for the oracle's own result rounded to bf16: what the output format alone costs
    floor = float(row_rel_err(f64(torch.from_numpy(want).to(torch.bfloat16)), want).max())
    # element by element against what the two bf16 storage formats of the path (H, Y) allow
    # (untimed; the oracle's FFN once more, with the variance of the H roundings beside it)
    mine, bound = layer_tokens_with_format_bound(orc, x, ids[toks], w[toks], keep, weights_of)
    worst = float((np.abs(got - want) / bound).max()) if np.allclose(mine, want, rtol=1e-12, atol=1e-300) else float("inf")
    local_rows = int(keep.any(axis=1).sum())
    above = int((row_err > ROW_TOL).sum())
    ints_ok = bool(np.array_equal(p.layer.buf.topk_ids.cpu().numpy(), ids)
                   and np.array_equal(p.layer.buf.inv.cpu().numpy()[: wl.T * wl.k], inv)
                   and np.array_equal(p.layer.buf.offsets.cpu().numpy()[: len(groups) + 1], offsets))
    yp_fp32 = p.layer.buf.Yp.dtype == torch.float32
    parity = bool(ints_ok and (not yp_fp32 or (worst <= 1.0 and above <= 1e-3 * max(local_rows, 1))))
    return dict(value=6.0 * wl.d * wl.f * rows / t_ffn / 1e12, unit="TFLOP/s", cores=_blas_threads(),
                host_cpus=os.cpu_count(), kind="oracle",
                sample=f"{wl.name}: every {stride}-th token ({len(toks)} tokens, {rows} local rows) through the "
                       f"fp64 per-token definition incl. widening {len(set(g[0] for g in groups))} experts' "
                       f"weights: {t_ffn:.1f} s; full routing+plan+permutation oracle (integer outputs): {t_int:.1f} s",
                seconds=t_ffn, integer_seconds=t_int, sample_max_row_err=err,
                sample_max_row_err_of_bf16_rounding_alone=floor, integer_outputs_match=ints_ok,
                row_bar=ROW_TOL, rows_checked=local_rows, rows_above_row_bar=above,
                worst_element_over_storage_format_bound=worst, parity=parity,
                parity_rule="integer outputs bit-equal; every element of Y inside the bound that bf16 H and bf16 Y "
                            "imply (half a bf16 step of the value + 7 sigma of the H roundings); at most 1 row in "
                            "1000 above 2e-2 of its RMS")


def _blas_threads():
    """Threads of the BLAS behind NumPy's matmul, which is where the oracle spends its time."""
    try:
        from threadpoolctl import threadpool_info
        n = [int(i["num_threads"]) for i in threadpool_info() if i.get("user_api") == "blas"]
        if n:
            return max(n)
    except Exception:
        pass
    import torch
    return torch.get_num_threads()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C4")
    ap.add_argument("--source", default="device", choices=["device", "pinned"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", "--no-c3", dest="only", action="store_true",
                    help="time the named workload only (default: the other four follow as short forward-only runs, reported under other_workloads)")
    ap.add_argument("--all", action="store_true", help="(kept for old command lines: all five workloads are the default now)")
    ap.add_argument("--cpu-tokens", type=int, default=65536)
    ap.add_argument("--no-training", action="store_true", help="skip the FFN training-step leg (forward keeping the SwiGLU derivatives, backward)")
    ap.add_argument("--yp-dtype", default="f32", choices=["f32", "bf16"],
                    help="type of the expert outputs Yp between the down GEMM and the combine")
    ap.add_argument("--plan-first", dest="early_static", action="store_false",
                    help="rebalanced share: read the counts back and plan before anything else is launched, one permute over all groups "
                         "(default: the timeline of Section 2.3 -- static experts launched before the plan is known, replicas' groups appended behind the static FFN)")
    ap.add_argument("--materialize-xp", action="store_true",
                    help="permute writes the permuted copy Xp and the gate/up GEMM reads it (default: the GEMM gathers the rows itself)")
    a = ap.parse_args()
    if a.gpus != 1:
        log("bench.py: this build is a single-GPU hot path (one EP rank's share); run it with --gpus 1")
        sys.exit(2)
    import torch
    import paper_2604_19654_amd as fe
    if not torch.cuda.is_available():
        log("bench.py needs a GPU")
        sys.exit(2)
    fe.lib()  # fail loudly if the HIP library is missing
    prop = torch.cuda.get_device_properties(0)
    p, res = time_workload(a.workload, a.steps, a.warmup, a.source, not a.materialize_xp, a.yp_dtype, a.early_static)
    log(json.dumps(res))
    cpu = None
    if not a.no_cpu_baseline:
        cpu = cpu_baseline(p, a.cpu_tokens)
    training = None
    if not a.no_training and res["f"] % 256 == 0 and res["d"] % 256 == 0:
        training = training_leg(p, a.steps)
        log(json.dumps(training))
        torch.cuda.empty_cache()
    # the other four workloads, each a short run of its own (forward step only): C3 is the other share the
    # grouped-FFN target names; C2, C5 and C1 complete the record
    others = {}
    p.wl.drop_weights()
    del p
    torch.cuda.empty_cache()
    for name in () if a.only else ("C3", "C2", "C5", "C1", "C4"):
        if name == a.workload:
            continue
        q, r = time_workload(name, a.steps, a.warmup, a.source, not a.materialize_xp, a.yp_dtype, a.early_static)
        log(json.dumps(r))
        others[name] = _summary(r)
        q.wl.drop_weights()
        del q
        torch.cuda.empty_cache()
    out = {
        "metric": METRIC, "value": res["ffn_tflops_step"], "unit": "TFLOP/s", "n_gpus": 1,
        "steps": a.steps, "warmup": a.warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{a.workload} ({_describe(a.workload)})", "T": res["T"], "R": res["R"],
                   "d": res["d"], "f": res["f"], "E": res["E"], "k": res["k"], "groups": res["groups"],
                   "nonempty_groups": res["nonempty_groups"],
                   "yp_dtype": a.yp_dtype, "x_rows": "permuted copy" if a.materialize_xp else "gathered by the gate/up GEMM",
                   "schedule": ("static experts launched before the plan" if a.early_static else "plan first") if a.workload == "C4" else None,
                   "staging_source": a.source if a.workload == "C4" else None},
        "roofline": res["rooflines"]["gate_up"],
        "rooflines": {k: v for k, v in res["rooflines"].items() if k != "gate_up"},
        "cpu_baseline": cpu,
        "ffn_training_step": training,
        "detail": {k: res[k] for k in res if k not in ("workload", "rooflines")},
        "device": _device_info(prop),
    }
    if others:
        out["other_workloads"] = others
    print(json.dumps(out), flush=True)


def _summary(r):
    """The figures of a secondary workload: step time, both GEMMs with their fraction of the MFMA peak, the
    bandwidth kernels with theirs."""
    rf = r["rooflines"]
    out = {k: r[k] for k in ("R", "nonempty_groups", "ms_per_step", "ffn_tflops_kernels", "pct_mfma_peak_ffn_kernels",
                             "graph_replay_ms_per_step") if k in r}
    for key in ("gate_up", "down"):
        out[key] = {"tflops": rf[key]["achieved"], "frac": rf[key]["frac"], "avg_launch_ms": rf[key]["avg_launch_ms"]}
    for key in ("combine", "permute_with_gather", "route"):
        out[key] = {"achieved": rf[key]["achieved"], "unit": rf[key]["unit"], "frac": rf[key]["frac"], "ms": rf[key]["avg_launch_ms"]}
    return out


def _device_info(prop):
    """CU count and clock as the runtime reports them, and the bf16 MFMA peak they imply
    (CUs x 4 SIMDs x 1024 flop/clk x clock); the published 2.5 PFLOP/s is what fractions use."""
    khz = getattr(prop, "clock_rate", None)
    if khz is None:
        try:
            import ctypes
            from paper_2604_19654_amd.binding import hip_runtime
            v = ctypes.c_int(0)
            # hipDeviceAttributeClockRate: peak clock in kHz
            hip = hip_runtime()
            hip.hipDeviceGetAttribute.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.c_int, ctypes.c_int]
            if hip.hipDeviceGetAttribute(ctypes.byref(v), 5, 0) == 0 and v.value > 0:
                khz = v.value
        except Exception:
            khz = None
    info = {"name": prop.name, "cus": prop.multi_processor_count, "hbm_gb": prop.total_memory / 2**30}
    if khz:
        info["clock_mhz"] = khz / 1e3
        info["derived_bf16_peak_tflops"] = prop.multi_processor_count * 4 * 1024 * khz * 1e3 / 1e12
    return info


def _describe(name):
    return {"C1": "tiny, 8 experts all local", "C2": "balanced rank share, EP=8",
            "C3": "skewed straggler share, EP=8", "C4": "FEPLB-rebalanced share: 16 static + 4 replicated experts",
            "C5": "large share, EP=4"}[name]


if __name__ == "__main__":
    main()
