"""The element-wise bound that the path's two bf16 storage formats imply (tests/util.py) against a
float64 computation that rounds exactly those two tensors, H and Y, and nothing else: the bound
must cover it with room to spare but not by orders of magnitude, and its parts must matter."""
import numpy as np
import torch

import workloads
from oracle import feplb_oracle as orc
from tests.util import (f64, bf16_half_ulp, format_bound, h_rounding_variance, layer_tokens_with_format_bound,
                        FORMAT_NSIGMA)


def bf16(x):
    return f64(torch.from_numpy(np.asarray(x, dtype=np.float64)).to(torch.float32).to(torch.bfloat16))


def test_half_ulp_is_the_rounding_radius_of_bf16():
    rng = np.random.default_rng(0)
    v = rng.normal(size=20000) * np.exp2(rng.integers(-20, 20, size=20000))
    err = np.abs(bf16(v.astype(np.float32)) - v.astype(np.float32))
    hu = bf16_half_ulp(v.astype(np.float32))
    assert (err <= hu).all()
    assert (err > 0.99 * hu).any()                      # and it is reached
    assert bf16_half_ulp(np.array([1.0]))[0] == 2.0 ** -8 and bf16_half_ulp(np.array([1.99]))[0] == 2.0 ** -8
    assert bf16_half_ulp(np.array([2.0]))[0] == 2.0 ** -7


def emulate(wl, toks, ids, w, keep, round_h=True, round_y=True):
    x = f64(wl.X)[toks]
    out = np.zeros_like(x)
    for e in sorted(set(int(v) for v in ids[toks][keep])):
        tok, slot = np.nonzero((ids[toks] == e) & keep)
        wg, wu, wd = (f64(m) for m in wl.expert_weights(e))
        h, _ = orc.ffn_rows(x[tok], wg, wu, wd)
        if round_h:
            h = bf16(h)
        out[tok] += w[toks][tok, slot][:, None] * (h @ wd)
    return bf16(out) if round_y else out


def test_bound_covers_a_computation_that_rounds_h_and_y_only():
    wl = workloads.make("C3", T=1024, d=512, f=256)
    ids, w, counts = orc.route_topk(f64(wl.logits).astype(np.float32), wl.k)
    local = set(int(e) for e in wl.local_experts())
    toks = np.arange(wl.T)
    keep = np.isin(ids, list(local))
    weights_of = lambda e: tuple(f64(m) for m in wl.expert_weights(e))
    want = orc.moe_tokens(f64(wl.X), ids, w, keep, weights_of)
    mine, bound = layer_tokens_with_format_bound(orc, f64(wl.X), ids, w, keep, weights_of)
    assert np.allclose(mine, want, rtol=1e-12, atol=1e-300)
    got = emulate(wl, toks, ids, w, keep)
    ratio = np.abs(got - want) / bound
    has = keep.any(axis=1)
    assert ratio.max() <= 1.0
    assert ratio[has].max() >= 0.5               # not a loose bound: the worst element uses most of it
    assert (bound[~has] <= 1e-29).all() and not got[~has].any()
    # the H term alone: Y kept unrounded; its error must stay inside n sigma and reach a good part of it
    got_h = emulate(wl, toks, ids, w, keep, round_y=False)
    only_h = np.abs(got_h - want)
    assert (only_h <= bound).all()
    rows = np.nonzero(has)[0]
    # measured spread of the H-rounding error against the sigma the bound is built from
    var = np.zeros_like(want)
    for e in sorted(set(int(v) for v in ids[keep])):
        tok, slot = np.nonzero((ids == e) & keep)
        _, _, v = h_rounding_variance(orc, f64(wl.X)[tok], weights_of(e))
        var[tok] += (w[tok, slot][:, None] ** 2) * v
    z = only_h[rows] / np.sqrt(var[rows])
    assert 0.6 <= np.sqrt((z ** 2).mean()) <= 1.2, np.sqrt((z ** 2).mean())     # sigma is the error's real scale
    assert z.max() <= FORMAT_NSIGMA
    # a bound without the combine weights, or without the output rounding, would be wrong
    got_y = emulate(wl, toks, ids, w, keep, round_h=False)
    assert (np.abs(got_y - want) <= bf16_half_ulp(want) * (1 + 1e-4) + 1e-30).all()      # (float64 -> fp32 -> bf16 rounds twice)
    assert (np.abs(got - want) > format_bound(want, var, output_bf16=False)).any()
