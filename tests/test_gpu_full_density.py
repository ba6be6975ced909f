"""Float parity at the benchmark's own sizes, densely: all five workloads in bench.py's launch
configuration, checked
  - on at least two permuted rows of EVERY 256-row tile of every group, for the activations H,
    the expert outputs Yp and the layer output Y of those rows' tokens, and
  - on every second token of the batch for Y (the sample bench.py's cpu_baseline leg uses; on every
    token of the three small workloads),
against the float64 oracle.  Every element must stay inside the bound that the path's two bf16
storage formats imply (tests/util.py, format_bound); rows on which that bound leaves room must
also meet the plain bar of 2e-2 of the row's RMS; the rows that exceed 2e-2 are counted (at most
one in a thousand may) and printed with the error that rounding the oracle's own result to bf16
causes on the same row.
Needs an MI355X: run with -m gpu."""
import numpy as np
import pytest
import torch

from paper_2604_19654_amd import runner
from oracle import feplb_oracle as orc
from tests.util import (f64, row_rel_err, bf16_rounding_excess, ROW_TOL, format_bound, h_rounding_variance,
                        layer_tokens_with_format_bound)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TILE = 256          # rows per tile of the grouped GEMM


def say(*a):
    print(*a, flush=True)


def oracle_indices(p):
    wl = p.wl
    ids, w, counts = orc.route_topk(wl.logits.cpu().numpy(), wl.k)
    if p.rebalanced:
        this = orc.pick_receiver(wl.P, wl.owner(), counts)
        moves, _, _ = orc.plan_overflow(wl.P, wl.owner(), counts, wl.dyn_flags(4), p.slots, this)
        groups = [(int(e), 0, orc.INT32_MAX) for e in wl.local_experts(this)] + [(m[0], m[4], m[4] + m[3]) for m in moves]
    else:
        groups = [(int(e), 0, orc.INT32_MAX) for e in wl.local_experts()]
    offsets, row_src, inv = orc.permute(ids, groups)
    return ids, w, groups, offsets, row_src, inv


def report_rows(tag, got, want, bound):
    """Element-wise format bound on every element; per-row figures; the rows above the plain bar."""
    err = np.abs(got - want)
    rms = np.sqrt((want ** 2).mean(axis=1))
    local = rms > 0
    assert not got[~local].any(), f"{tag}: a token without a local slot is not exactly zero"
    worst = float((err / bound).max())
    row_err = np.zeros(len(want)); row_bound = np.zeros(len(want)); row_floor = np.zeros(len(want))
    row_err[local] = err[local].max(axis=1) / rms[local]
    row_bound[local] = bound[local].max(axis=1) / rms[local]
    rounded = f64(torch.from_numpy(want[local]).to(torch.bfloat16))
    row_floor[local] = np.abs(rounded - want[local]).max(axis=1) / rms[local]
    over = np.nonzero(row_err > ROW_TOL)[0]
    say(f"  {tag}: {int(local.sum())} rows with local work; per-row max-abs error / row RMS: max {row_err.max():.4f}, "
        f"99.9th percentile {np.quantile(row_err[local], 0.999):.4f}, median {np.median(row_err[local]):.4f}; "
        f"largest element error / format bound {worst:.3f}")
    say(f"  {tag}: {len(over)} rows above {ROW_TOL} ({100.0 * len(over) / max(1, int(local.sum())):.4f} %), "
        f"largest excess {max(0.0, row_err.max() - ROW_TOL):.4f}")
    for r in over[np.argsort(-row_err[over])][:12]:
        say(f"    row {r}: error {row_err[r]:.4f}, bf16 rounding of the oracle's row alone {row_floor[r]:.4f}, "
            f"format bound of the row {row_bound[r]:.4f}")
    assert worst <= 1.0, f"{tag}: an element is outside the bound of the storage formats ({worst:.3f} of it)"
    room = local & (row_bound <= ROW_TOL)
    say(f"  {tag}: the format bound leaves room under {ROW_TOL} on {int(room.sum())} rows "
        f"(median row bound {np.median(row_bound[local]):.4f}, largest {row_bound.max():.4f})")
    assert (row_err[room] <= ROW_TOL).all()
    # the rest may pass 2e-2 only as rare tail events of the H roundings (measured: 1 row in 26 647 on the
    # rebalanced share); a systematic extra rounding would put whole percents of the rows above it
    assert len(over) <= 1e-3 * local.sum(), f"{tag}: {len(over)} rows above {ROW_TOL}"
    return row_err, row_floor


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_every_tile_and_every_second_token_at_full_size(name):
    say(f"layer {name} at full size, launch configuration of the benchmark")
    p = runner.prepare(name, DEV)
    Y = runner.step(p)
    torch.cuda.synchronize()
    wl, b = p.wl, p.layer.buf
    ids, w, groups, offsets, row_src, inv = oracle_indices(p)
    G, R = len(groups), int(offsets[-1])
    assert np.array_equal(b.offsets.cpu().numpy()[: G + 1], offsets) and np.array_equal(b.inv.cpu().numpy()[: wl.T * wl.k], inv)
    assert np.array_equal(b.row_src.cpu().numpy()[:R], row_src)
    weights_of = lambda e: tuple(f64(m) for m in wl.expert_weights(e))

    # ---- two rows of every tile (three where the tile has them: first, last, one inside)
    rng = np.random.default_rng(7)
    rows, row_group = [], []
    n_tiles = 0
    for g in range(G):
        for lo in range(int(offsets[g]), int(offsets[g + 1]), TILE):
            hi = min(lo + TILE, int(offsets[g + 1]))
            pick = {lo, hi - 1, int(rng.integers(lo, hi))}
            if hi - lo >= 2:
                assert len(pick) >= 2
            rows += sorted(pick)
            row_group += [g] * len(pick)
            n_tiles += 1
    rows, row_group = np.array(rows), np.array(row_group)
    say(f"  {name}: R={R}, {n_tiles} tiles in {int((np.diff(offsets) > 0).sum())} non-empty groups, {len(rows)} rows sampled")
    rows_dev = torch.from_numpy(rows).to(DEV)
    x_rows = f64(wl.X[torch.from_numpy(row_src[rows].astype(np.int64) // wl.k).to(DEV)])
    H_got, Yp_got = f64(b.H[rows_dev]), f64(b.Yp[rows_dev])
    H_want = np.zeros_like(H_got); Yp_want = np.zeros_like(Yp_got); Yp_var = np.zeros_like(Yp_got)
    for g in sorted(set(row_group.tolist())):
        sel = np.nonzero(row_group == g)[0]
        H_want[sel], Yp_want[sel], Yp_var[sel] = h_rounding_variance(orc, x_rows[sel], weights_of(groups[g][0]))
    h_excess = bf16_rounding_excess(H_got, H_want)
    yp_bound = format_bound(Yp_want, Yp_var, output_bf16=False)
    yp_worst = float((np.abs(Yp_got - Yp_want) / yp_bound).max())
    yp_row = row_rel_err(Yp_got, Yp_want)
    say(f"  {name} tiles: H largest error / (one bf16 step + 1e-3 row RMS) {h_excess:.3f}; Yp largest element error / "
        f"format bound {yp_worst:.3f}, per-row error max {yp_row.max():.4f} (bound {ROW_TOL})")
    assert h_excess <= 1.0
    assert yp_worst <= 1.0
    assert yp_row.max() <= ROW_TOL          # fp32 expert outputs: no output rounding, the plain bar holds
    toks = np.unique(row_src[rows] // wl.k)
    keep = inv.reshape(wl.T, wl.k)[toks] >= 0
    toks_dev = torch.from_numpy(toks).to(DEV)
    want = orc.moe_tokens(f64(wl.X[toks_dev]), ids[toks], w[toks], keep, weights_of)
    mine, bound = layer_tokens_with_format_bound(orc, f64(wl.X[toks_dev]), ids[toks], w[toks], keep, weights_of)
    assert np.allclose(mine, want, rtol=1e-12, atol=1e-300)
    report_rows(f"{name} Y of the tile rows' tokens", f64(Y[toks_dev]), want, bound)

    # ---- every second token of the batch (every token of the three small workloads)
    toks = np.arange(0, wl.T, 2 if wl.T > 16384 else 1)
    keep = inv.reshape(wl.T, wl.k)[toks] >= 0
    toks_dev = torch.from_numpy(toks).to(DEV)
    x = f64(wl.X[toks_dev])
    want = orc.moe_tokens(x, ids[toks], w[toks], keep, weights_of)
    mine, bound = layer_tokens_with_format_bound(orc, x, ids[toks], w[toks], keep, weights_of)
    assert np.allclose(mine, want, rtol=1e-12, atol=1e-300)
    del mine, x
    report_rows(f"{name} Y of {len(toks)} of {wl.T} tokens", f64(Y[toks_dev]), want, bound)
    p.wl.drop_weights()
    torch.cuda.empty_cache()
