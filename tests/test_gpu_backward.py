"""Parity of the HIP backward pass of the grouped expert FFN with the CPU oracle, through the
C ABI.  The oracle differentiates the float64 definition; the library keeps its activations and
their gradients in bf16, so every output row is held to BWD_RMS_TOL (root-mean-square error) and
BWD_MAX_TOL (largest error) of that row's RMS; tests/util.py derives both bars.  Beside each result the tests print what a float64
computation that merely stores p, q, H, da, db in bf16 would get: a diagnostic, not a bound.
Needs an MI355X: run with -m gpu."""
import numpy as np
import pytest
import torch

import paper_2604_19654_amd as fe
from paper_2604_19654_amd import binding as B
from oracle import feplb_oracle as orc
from tests.util import (f64, row_rel_err, row_rms_err, bf16_rounding_excess, BWD_RMS_TOL, BWD_MAX_TOL, FORMAT_NSIGMA,
                        h_rounding_variance)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


def make_weights(G, d, f, seed):
    g = torch.Generator().manual_seed(seed)
    return [tuple((torch.randn(s, generator=g) * 0.05).to(torch.bfloat16) for s in ((d, f), (d, f), (f, d)))
            for _ in range(G)]


def run_forward_backward(sizes, d, f, dxp_dtype, pad=37, seed=7, poison=float("nan")):
    """One training step of the library on groups of the given sizes; rows past R hold `poison`."""
    G = len(sizes)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    R = int(offsets[-1])
    R_cap = max(R + pad, 32)
    gen = torch.Generator().manual_seed(seed)
    Xp = torch.randn((R_cap, d), generator=gen).to(torch.bfloat16)
    dYp = torch.randn((R_cap, d), generator=gen).to(torch.bfloat16)
    Xp[R:] = poison
    dYp[R:] = poison
    W = make_weights(G, d, f, seed + 4)
    Wd = [tuple(m.to(DEV) for m in w) for w in W]
    H = torch.full((R_cap, f), poison, dtype=torch.bfloat16, device=DEV)
    AB = torch.full((R_cap, 2 * f), poison, dtype=torch.bfloat16, device=DEV)
    Yp = torch.full((R_cap, d), 512.0, dtype=torch.float32, device=DEV)
    dXp = torch.full((R_cap, d), 512.0, dtype=dxp_dtype, device=DEV)
    off_dev = torch.from_numpy(offsets).to(DEV)
    Xp_dev, dYp_dev = Xp.to(DEV), dYp.to(DEV)
    wg, wu, wd = ([w[i] for w in Wd] for i in range(3))
    fe.feplb_grouped_ffn(Xp_dev, off_dev, 0, G, d, f, wg, wu, wd, H, Yp, AB=AB)
    torch.cuda.synchronize()
    AB_saved = AB.clone()
    dW = [tuple(torch.full(s, 7.0, dtype=torch.float32, device=DEV) for s in ((d, f), (d, f), (f, d))) for _ in range(G)]
    B.feplb_grouped_ffn_backward(Xp_dev, off_dev, 0, G, d, f, wg, wu, wd, H, AB, dYp_dev, dXp,
                                 [w[0] for w in dW], [w[1] for w in dW], [w[2] for w in dW])
    torch.cuda.synchronize()
    return dict(offsets=offsets, R=R, R_cap=R_cap, Xp=Xp, dYp=dYp, W=W, H=H, AB_saved=AB_saved, dAB=AB, Yp=Yp,
                dXp=dXp, dW=dW)


def oracle_backward(r):
    R = r["R"]
    Wo = [tuple(f64(m) for m in w) for w in r["W"]]
    return orc.grouped_ffn_backward(f64(r["Xp"])[:R], r["offsets"], Wo, f64(r["dYp"])[:R]), Wo


def bf16_round(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(torch.bfloat16).to(torch.float64).numpy()


def storage_format_floor(r, dXp_o, grads_o, Wo):
    """Worst row error of a float64 backward whose only inexactness is keeping p, q, H, da, db in
    bf16 (diagnostic printed beside the library's figures)."""
    R = r["R"]
    X, dY = f64(r["Xp"])[:R], f64(r["dYp"])[:R]
    worst = np.zeros(4)     # dXp rms, dXp max, weights rms, weights max
    for g, (wg, wu, wd) in enumerate(Wo):
        lo, hi = int(r["offsets"][g]), int(r["offsets"][g + 1])
        if hi == lo:
            continue
        x, dy = X[lo:hi], dY[lo:hi]
        a0, b0 = x @ wg, x @ wu
        h = bf16_round(a0 / (1.0 + np.exp(-a0)) * b0)
        sg = 1.0 / (1.0 + np.exp(-a0))
        dp, dq = bf16_round(b0 * sg * (1.0 + a0 * (1.0 - sg))), bf16_round(a0 * sg)
        dh = dy @ wd.T
        da, db = bf16_round(dh * dp), bf16_round(dh * dq)
        dx = da @ wg.T + db @ wu.T
        worst[0] = max(worst[0], row_rms_err(dx, dXp_o[lo:hi]).max())
        worst[1] = max(worst[1], row_rel_err(dx, dXp_o[lo:hi]).max())
        for got, want in zip((x.T @ da, x.T @ db, h.T @ dy), grads_o[g]):
            worst[2] = max(worst[2], row_rms_err(got, want).max())
            worst[3] = max(worst[3], row_rel_err(got, want).max())
    return "bf16 storage alone: dXp rms %.5f max %.5f, weights rms %.5f max %.5f" % tuple(worst)


def check_rows(got, want, what):
    """Both bars on every row; returns (worst rms error, worst largest error)."""
    e_rms, e_max = row_rms_err(got, want), row_rel_err(got, want)
    assert e_rms.max() <= BWD_RMS_TOL, f"{what}: rms error {e_rms.max():.5f} of the row RMS"
    assert e_max.max() <= BWD_MAX_TOL, f"{what}: largest error {e_max.max():.5f} of the row RMS"
    return float(e_rms.max()), float(e_max.max())


def check_weight_grads(r, grads_o, label):
    worst = (0.0, 0.0)
    for g, (got3, want3) in enumerate(zip(r["dW"], grads_o)):
        rows = int(r["offsets"][g + 1] - r["offsets"][g])
        for got, want, name in zip(got3, want3, ("dW_gate", "dW_up", "dW_down")):
            gv = f64(got)
            if rows == 0:
                assert not gv.any(), f"{label}: {name}[{g}] of an empty group is not zero"
                continue
            e = check_rows(gv, want, f"{label}: {name}[{g}] ({rows} rows)")
            worst = (max(worst[0], e[0]), max(worst[1], e[1]))
    return worst


@pytest.mark.parametrize("sizes,d,f", [([128, 0, 1, 129, 300, 0, 64, 255], 256, 256),
                                       ([5, 700], 512, 256), ([0, 0, 0], 256, 256), ([1], 768, 256),
                                       ([3], 256, 256), ([33, 31, 32, 64, 65], 256, 512),
                                       ([0, 40, 0], 256, 256)])
@pytest.mark.parametrize("dxp_dtype", [torch.float32, torch.bfloat16])
def test_grouped_ffn_backward_parity(sizes, d, f, dxp_dtype):
    say(f"ffn backward sizes={sizes} d={d} f={f} {dxp_dtype}")
    r = run_forward_backward(sizes, d, f, dxp_dtype)
    R = r["R"]
    (dXp_o, grads_o), Wo = oracle_backward(r)
    if R:
        # what the forward kept: the derivatives p = dH/da, q = dH/db of the SwiGLU product,
        # within a bf16 rounding step of their float64 values
        X64 = f64(r["Xp"])[:R]
        p_o = np.zeros((R, f)); q_o = np.zeros((R, f))
        for g in range(len(sizes)):
            lo, hi = int(r["offsets"][g]), int(r["offsets"][g + 1])
            a_g, b_g = X64[lo:hi] @ Wo[g][0], X64[lo:hi] @ Wo[g][1]
            s_g = 1.0 / (1.0 + np.exp(-a_g))
            p_o[lo:hi] = b_g * s_g * (1.0 + a_g * (1.0 - s_g))
            q_o[lo:hi] = a_g * s_g
        ea = bf16_rounding_excess(f64(r["AB_saved"])[:R, :f], p_o)
        eb = bf16_rounding_excess(f64(r["AB_saved"])[:R, f:], q_o)
        ex = check_rows(f64(r["dXp"])[:R], dXp_o, "dXp")
        say(f"  saved p, q rounding excess {ea:.3f} {eb:.3f} (<= 1)  dXp rms {ex[0]:.5f} max {ex[1]:.5f}")
        assert ea <= 1.0 and eb <= 1.0
    worst = check_weight_grads(r, grads_o, "parity")
    say(f"  weight gradients rms {worst[0]:.5f} max {worst[1]:.5f} (<= {BWD_RMS_TOL}, {BWD_MAX_TOL})")
    say("  " + storage_format_floor(r, dXp_o, grads_o, Wo))
    # rows past R are never written
    assert (r["dXp"][R:].float() == 512.0).all()
    assert torch.isnan(r["dAB"][R:].float()).all() and torch.isnan(r["H"][R:].float()).all()


def test_grouped_ffn_backward_larger_ragged_case_and_repeatability():
    # several row tiles per group, contraction tails of every residue class, f != d
    sizes = [517, 2, 1031, 0, 255, 770, 96, 1]
    d, f = 1024, 768
    say(f"ffn backward sizes={sizes} d={d} f={f}")
    r = run_forward_backward(sizes, d, f, torch.float32, poison=512.0)
    (dXp_o, grads_o), Wo = oracle_backward(r)
    ex = check_rows(f64(r["dXp"])[:r["R"]], dXp_o, "dXp")
    worst = check_weight_grads(r, grads_o, "larger")
    say(f"  dXp rms {ex[0]:.5f} max {ex[1]:.5f}  weight gradients rms {worst[0]:.5f} max {worst[1]:.5f}")
    say("  " + storage_format_floor(r, dXp_o, grads_o, Wo))
    r2 = run_forward_backward(sizes, d, f, torch.float32, poison=512.0)
    assert torch.equal(r["dXp"], r2["dXp"]) and torch.equal(r["dAB"], r2["dAB"])
    for a3, b3 in zip(r["dW"], r2["dW"]):
        assert all(torch.equal(a, b) for a, b in zip(a3, b3))


def test_grouped_ffn_backward_refuses_bad_arguments():
    d = f = 256
    z = torch.zeros((64, d), dtype=torch.bfloat16, device=DEV)
    ab = torch.zeros((64, 2 * f), dtype=torch.bfloat16, device=DEV)
    off = torch.tensor([0, 64], dtype=torch.int32, device=DEV)
    w = [torch.zeros((d, f), dtype=torch.bfloat16, device=DEV)]
    dw = [torch.zeros((d, f), dtype=torch.float32, device=DEV)]
    dx = torch.zeros((64, d), dtype=torch.float32, device=DEV)
    with pytest.raises(B.FeplbError):      # f not a multiple of 256
        B.feplb_grouped_ffn_backward(z, off, 0, 1, d, 128, w, w, w, z, ab, z, dx, dw, dw, dw)
    with pytest.raises(B.FeplbError):      # scratch for the transposed weights too small
        B.feplb_grouped_ffn_backward(z, off, 0, 1, d, f, w, w, w, z, ab, z, dx, dw, dw, dw,
                                     WT=torch.zeros((1024,), dtype=torch.uint8, device=DEV))
    small = torch.zeros((16, d), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.FeplbError):      # fewer than 32 rows of capacity for the weight gradients
        B.feplb_grouped_ffn_backward(small, off, 0, 1, d, f, w, w, w, small, ab[:16], small, dx[:16], dw, dw, dw)
    torch.cuda.synchronize()


def test_weight_gradients_add_up_over_a_split_of_the_rows():
    # one group of n rows against the same rows as two groups with the same matrices: da | db
    # are computed row by row, so the gradients must agree up to the order of the fp32 sums --
    # far below the float bar, and sensitive to every row at a window or group boundary
    d, f = 256, 256
    for n, cut in [(100, 37), (64, 32), (45, 1), (300, 257), (31, 30)]:
        say(f"ffn backward split n={n} cut={cut}")
        gen = torch.Generator().manual_seed(n)
        Xp = torch.randn((n + 50, d), generator=gen).to(torch.bfloat16).to(DEV)
        dYp = torch.randn((n + 50, d), generator=gen).to(torch.bfloat16).to(DEV)
        w = make_weights(1, d, f, 3)[0]
        w = tuple(m.to(DEV) for m in w)
        res = []
        for sizes in ([n], [cut, n - cut]):
            G = len(sizes)
            off = torch.tensor(np.concatenate([[0], np.cumsum(sizes)]), dtype=torch.int32, device=DEV)
            H = torch.zeros((n + 50, f), dtype=torch.bfloat16, device=DEV)
            AB = torch.zeros((n + 50, 2 * f), dtype=torch.bfloat16, device=DEV)
            Yp = torch.zeros((n + 50, d), dtype=torch.float32, device=DEV)
            dXp = torch.zeros((n + 50, d), dtype=torch.float32, device=DEV)
            wl = [[w[i]] * G for i in range(3)]
            dW = [[torch.zeros(s, dtype=torch.float32, device=DEV) for _ in range(G)] for s in ((d, f), (d, f), (f, d))]
            fe.feplb_grouped_ffn(Xp, off, 0, G, d, f, *wl, H, Yp, AB=AB)
            B.feplb_grouped_ffn_backward(Xp, off, 0, G, d, f, *wl, H, AB, dYp, dXp, *dW)
            torch.cuda.synchronize()
            res.append((dXp, [sum(m.double() for m in mats) for mats in dW]))
        assert torch.equal(res[0][0], res[1][0])
        for one, two in zip(res[0][1], res[1][1]):
            scale = one.pow(2).mean().sqrt().item()
            assert (one - two).abs().max().item() <= 1e-5 * scale


@pytest.mark.parametrize("name", ["C3", "C4", "C5"])
def test_backward_at_full_size_on_sampled_outputs(name):
    """The training step in the configuration bench.py times (the workload's own groups and token
    rows, all groups in one call), checked where the oracle can follow: dXp on sampled rows (a row
    needs only its own x and dy), weight gradients on sampled columns of sampled groups (a column
    of dWg, dWu needs that column of da, db for every row of the group; a column of dWd needs that
    column of dYp)."""
    from paper_2604_19654_amd import runner
    from paper_2604_19654_amd.training import setup_from_prepared
    say(f"backward {name} at full size")
    p = runner.prepare(name, DEV)
    runner.step(p)
    torch.cuda.synchronize()
    st, Xp, offsets, (wg, wu, wd), dYp = setup_from_prepared(p)
    st.forward(Xp, offsets, wg, wu, wd)
    st.backward(Xp, offsets, wg, wu, wd, dYp)
    torch.cuda.synchronize()
    off = offsets.cpu().numpy()
    sizes = np.diff(off)
    say(f"  groups {sizes.tolist()}")
    order = np.argsort(-sizes, kind="stable")
    picked = [int(order[0]), int(order[min(2, len(order) - 1)])] + [int(g) for g in order if 0 < sizes[g] < 64][:2]
    worst = np.zeros(4)
    for g in dict.fromkeys(picked):
        lo, hi = int(off[g]), int(off[g + 1])
        if hi == lo:
            continue
        Wg, Wu, Wd = f64(wg[g]), f64(wu[g]), f64(wd[g])
        rows = np.unique(np.concatenate([[lo, hi - 1], np.arange(lo, hi, max(1, (hi - lo) // 6))]))
        dx_o = orc.ffn_rows_backward(f64(Xp[rows]), Wg, Wu, Wd, f64(dYp[rows]))[0]
        e = check_rows(f64(st.dXp[rows]), dx_o, f"{name}: dXp rows of group {g}")
        worst[:2] = np.maximum(worst[:2], e)
        # Sampled columns through the oracle itself.  The expert is separable over its hidden units
        # (y = sum_j h_j Wd[j,:]), so the oracle run on the sub-expert made of hidden units `cols`
        # (Wg[:, cols], Wu[:, cols], Wd[cols, :]) with the same dy returns exactly the columns `cols` of
        # dWg and dWu; and run on the output columns `dcols` alone (Wd[:, dcols], dy[:, dcols]) it returns
        # exactly those columns of dWd.  (One row per sampled column below.)
        cols = [0, st.f // 2 + 1, st.f - 1]
        X64, dY64 = f64(Xp[lo:hi]), f64(dYp[lo:hi])
        _, dWg_c, dWu_c, _ = orc.ffn_rows_backward(X64, Wg[:, cols], Wu[:, cols], Wd[cols, :], dY64)
        e = check_rows(f64(st.dW_gate[g][:, cols]).T, dWg_c.T, f"{name}: dW_gate[{g}] columns")
        worst[2:] = np.maximum(worst[2:], e)
        e = check_rows(f64(st.dW_up[g][:, cols]).T, dWu_c.T, f"{name}: dW_up[{g}] columns")
        worst[2:] = np.maximum(worst[2:], e)
        dcols = [0, st.d // 2 + 1, st.d - 1]
        dWd_c = orc.ffn_rows_backward(X64, Wg, Wu, Wd[:, dcols], dY64[:, dcols])[3]
        e = check_rows(f64(st.dW_down[g][:, dcols]).T, dWd_c.T, f"{name}: dW_down[{g}] columns")
        worst[2:] = np.maximum(worst[2:], e)
        say(f"  group {g} ({hi - lo} rows) checked")
    for g in np.nonzero(sizes == 0)[0][:3]:
        assert not st.dW_gate[g].any() and not st.dW_up[g].any() and not st.dW_down[g].any()
    # the same step again, several times: every output bit for bit (counted waits of the
    # pipelines leave no room for a load that lands late)
    big = int(order[0])
    ref = (st.dXp.clone(), st.AB.clone(), st.dW_gate[big].clone(), st.dW_down[big].clone())
    for _ in range(4):
        st.forward(Xp, offsets, wg, wu, wd)
        st.backward(Xp, offsets, wg, wu, wd, dYp)
        torch.cuda.synchronize()
        now = (st.dXp, st.AB, st.dW_gate[big], st.dW_down[big])
        assert all(torch.equal(a_, b_) for a_, b_ in zip(ref, now)), "training step is not repeatable"
    say(f"  dXp rms {worst[0]:.5f} max {worst[1]:.5f}; weight gradients rms {worst[2]:.5f} max {worst[3]:.5f}")
    p.wl.drop_weights()
    torch.cuda.empty_cache()


def test_backward_of_a_split_group_range_equals_one_call():
    # static range, then dynamic range, as the forward pass is launched; outputs must be the same bits
    sizes = [300, 0, 45, 513, 70]
    d, f, cut = 512, 256, 3
    G = len(sizes)
    off = torch.tensor(np.concatenate([[0], np.cumsum(sizes)]), dtype=torch.int32, device=DEV)
    R = int(sum(sizes))
    gen = torch.Generator().manual_seed(21)
    Xp = torch.randn((R, d), generator=gen).to(torch.bfloat16).to(DEV)
    dYp = torch.randn((R, d), generator=gen).to(torch.bfloat16).to(DEV)
    W = [tuple(m.to(DEV) for m in w) for w in make_weights(G, d, f, 5)]
    wl = [[w[i] for w in W] for i in range(3)]
    res = []
    for ranges in ([(0, G)], [(0, cut), (cut, G)]):
        H = torch.zeros((R, f), dtype=torch.bfloat16, device=DEV)
        AB = torch.zeros((R, 2 * f), dtype=torch.bfloat16, device=DEV)
        Yp = torch.zeros((R, d), dtype=torch.float32, device=DEV)
        dXp = torch.zeros((R, d), dtype=torch.float32, device=DEV)
        dW = [[torch.full(s, 3.0, dtype=torch.float32, device=DEV) for _ in range(G)] for s in ((d, f), (d, f), (f, d))]
        for g0, g1 in ranges:
            fe.feplb_grouped_ffn(Xp, off, g0, g1, d, f, *wl, H, Yp, AB=AB)
        for g0, g1 in ranges:
            B.feplb_grouped_ffn_backward(Xp, off, g0, g1, d, f, *wl, H, AB, dYp, dXp, *dW)
        torch.cuda.synchronize()
        res.append((dXp, AB, dW))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])
    for mats_a, mats_b in zip(res[0][2], res[1][2]):
        assert all(torch.equal(a, b) for a, b in zip(mats_a, mats_b))


# ------------------------------------------------------------------ combine, row gather, router: backward
@pytest.mark.parametrize("T,k,d,yp_dtype", [(100, 2, 256, torch.float32), (333, 8, 520, torch.float32),
                                            (64, 4, 6144, torch.float32), (257, 8, 1024, torch.bfloat16), (5, 1, 8, torch.float32)])
def test_combine_backward_parity(T, k, d, yp_dtype):
    say(f"combine backward T={T} k={k} d={d} {yp_dtype}")
    rng = np.random.default_rng(T + d)
    n = T * k
    R = int(0.6 * n)
    inv = np.full(n, -1, dtype=np.int32)
    slots = rng.permutation(n)[:R]
    inv[slots] = rng.permutation(R)
    gen = torch.Generator().manual_seed(T)
    Yp = torch.randn((R + 5, d), generator=gen).to(yp_dtype)
    dY = torch.randn((T, d), generator=gen).to(torch.bfloat16)
    w = torch.rand((T, k), generator=gen) + 0.05
    dYp = torch.full((R + 5, d), 512.0, dtype=torch.bfloat16, device=DEV)
    _, dw = B.feplb_combine_backward(dY.to(DEV), Yp.to(DEV), torch.from_numpy(inv).to(DEV), w.to(DEV), T, k, d, dYp)
    torch.cuda.synchronize()
    dYp_o, dw_o = orc.combine_backward(f64(dY), f64(Yp)[:R], inv, f64(w), T, k)
    # dYp: one rounding of an fp32 product to bf16
    assert bf16_rounding_excess(f64(dYp)[:R], dYp_o) <= 1.0
    assert (dYp[R:].float() == 512.0).all()
    # dw: an fp32 dot product of d terms against the Cauchy-Schwarz scale of its two rows
    scale = np.zeros((T, k))
    inv2 = inv.reshape(T, k)
    for j in range(k):
        sel = inv2[:, j] >= 0
        scale[sel, j] = np.linalg.norm(f64(dY)[sel], axis=1) * np.linalg.norm(f64(Yp)[inv2[sel, j]], axis=1)
    err = np.abs(f64(dw) - dw_o)
    assert (err <= 1e-5 * scale + 1e-30).all(), err.max()
    assert not f64(dw)[inv2 < 0].any()


def test_permute_backward_is_the_combine_with_unit_weights():
    T, E, k, d = 300, 16, 4, 264
    rng = np.random.default_rng(8)
    ids = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    groups = [(e, 0, B.ORD_MAX) for e in (1, 4, 9, 15)]
    X = torch.zeros((T, d), dtype=torch.bfloat16, device=DEV)
    R_cap = T * k
    _, offsets, row_src, inv = B.feplb_permute(torch.from_numpy(ids).to(DEV), E, groups, None, R_cap)
    torch.cuda.synchronize()
    R = int(offsets[-1].item())
    dXp = torch.randn((R_cap, d), generator=torch.Generator().manual_seed(2)).to(DEV)
    dX = B.feplb_unpermute_combine(dXp, inv, torch.ones((T, k), device=DEV), T, k, d)
    torch.cuda.synchronize()
    want = orc.permute_backward(f64(dXp)[:R], inv.cpu().numpy(), T, k)
    # fp32 sums of at most k rows, one rounding to bf16: every element within a bf16 step
    assert bf16_rounding_excess(f64(dX), want) <= 1.0


@pytest.mark.parametrize("T,E,k", [(200, 8, 2), (1000, 128, 8), (77, 5, 5), (3, 1024, 32)])
def test_route_backward_parity(T, E, k):
    say(f"route backward T={T} E={E} k={k}")
    gen = torch.Generator().manual_seed(T + E)
    logits = torch.randn((T, E), generator=gen)
    dw = torch.randn((T, k), generator=gen)
    ids, w, _ = B.feplb_route_topk(logits.to(DEV), k)
    dz = B.feplb_route_topk_backward(ids, w, dw.to(DEV), E)
    torch.cuda.synchronize()
    want = orc.route_topk_backward(logits.numpy(), ids.cpu().numpy(), f64(dw))
    assert np.abs(f64(dz) - want).max() <= 2e-6 * max(1.0, float(dw.abs().max()))
    assert np.array_equal(f64(dz) != 0, want != 0) or np.abs(f64(dz) - want).max() < 1e-12


# ------------------------------------------------------------------ the layer's backward pass, end to end
LAYER_CASES = {
    "C1": {},                                     # the tiny workload at its full size (f=512, d=256)
    "C3": dict(T=2048, d=512, f=256),             # hot groups of ~2k rows, several empty groups
    "C5": dict(T=2048, d=768, f=256),             # 32 groups
}


@pytest.mark.parametrize("name", list(LAYER_CASES))
def test_layer_backward_parity(name):
    """Route, permute, training forward and combine, then the whole backward chain, against the
    oracle's chain on the same inputs: dX and the weight gradients per row, dlogits over all tokens."""
    from paper_2604_19654_amd import runner
    from paper_2604_19654_amd.training import setup_from_prepared, LayerBackward
    say(f"layer backward {name} {LAYER_CASES[name]}")
    p = runner.prepare(name, DEV, **LAYER_CASES[name])
    runner.step(p)
    torch.cuda.synchronize()
    wl, b = p.wl, p.layer.buf
    st, Xp, offsets, weights, _ = setup_from_prepared(p)
    st.forward(Xp, offsets, *weights)
    dY = torch.randn((wl.T, wl.d), generator=torch.Generator().manual_seed(17)).to(torch.bfloat16)
    lb = LayerBackward(wl.T, wl.E, wl.k, st)
    dX, dlogits = lb.run(dY.to(DEV), Xp, offsets, weights, b.topk_ids, b.topk_w, b.inv)
    torch.cuda.synchronize()

    ids, w, _ = orc.route_topk(wl.logits.cpu().numpy(), wl.k)
    groups = [(int(e), 0, orc.INT32_MAX) for e in wl.local_experts()]
    off_o, row_src, inv = orc.permute(ids, groups)
    R = int(off_o[-1])
    Wo = [tuple(f64(m) for m in wl.expert_weights(e)) for (e, _lo, _hi) in groups]
    Xp_o = orc.gather_rows(f64(wl.X), row_src, wl.k)
    _, Yp_o = orc.grouped_ffn(Xp_o, off_o, Wo)
    dYp_o, dw_o = orc.combine_backward(f64(dY), Yp_o, inv, w, wl.T, wl.k)
    dXp_o, grads_o = orc.grouped_ffn_backward(Xp_o, off_o, Wo, dYp_o)
    dX_o = orc.permute_backward(dXp_o, inv, wl.T, wl.k)
    dz_o = orc.route_topk_backward(wl.logits.cpu().numpy(), ids, dw_o)

    local = (inv.reshape(wl.T, wl.k) >= 0).any(axis=1)
    assert not f64(dX)[~local].any()                     # tokens without a local slot get no gradient
    ex = check_rows(f64(dX)[local], dX_o[local], "dX")
    r = dict(offsets=off_o, dW=list(zip(st.dW_gate, st.dW_up, st.dW_down)))
    ew = check_weight_grads(r, grads_o, "layer")
    # dlogits: the dot products behind dw cancel heavily, so single entries can be off by much more
    # than their own size and a bar relative to the entry makes no sense.  What an entry may be off by
    # follows from the storage formats: Yp carries the roundings of the bf16 activations H (variance
    # per element as in tests/util.py), so dw[t,j] = <dY[t,:], Yp[r,:]> carries a sum of them with
    # variance s2[t,j] = sum_i dY[t,i]^2 var(Yp[r,i]); the router's backward is linear in dw,
    # dz_j = w_j ((1 - w_j) dw_j - sum_{i != j} w_i dw_i), which gives each entry's variance; fp32
    # accumulation of the d-term dot product adds at most 1e-5 of the Cauchy-Schwarz scale of its rows.
    dz = f64(dlogits)
    rel = np.sqrt(((dz - dz_o) ** 2).mean()) / np.sqrt((dz_o ** 2).mean())
    yp_var = np.zeros_like(Yp_o)
    for g in range(len(groups)):
        lo, hi = int(off_o[g]), int(off_o[g + 1])
        if hi > lo:
            yp_var[lo:hi] = h_rounding_variance(orc, Xp_o[lo:hi], Wo[g])[2]
    inv2 = inv.reshape(wl.T, wl.k)
    s2 = np.zeros((wl.T, wl.k)); cs = np.zeros((wl.T, wl.k))
    dYo = f64(dY)
    for j in range(wl.k):
        sel = np.nonzero(inv2[:, j] >= 0)[0]
        s2[sel, j] = np.einsum("ij,ij->i", dYo[sel] ** 2, yp_var[inv2[sel, j]])
        cs[sel, j] = 1e-5 * np.linalg.norm(dYo[sel], axis=1) * np.linalg.norm(Yp_o[inv2[sel, j]], axis=1)
    var_dz = w ** 2 * ((1.0 - 2.0 * w) * s2 + (w ** 2 * s2).sum(axis=1, keepdims=True))      # (1-w_j)^2 s_j^2 + sum_{i!=j} w_i^2 s_i^2
    slack = w * ((1.0 - 2.0 * w) * cs + (w * cs).sum(axis=1, keepdims=True))
    bound = FORMAT_NSIGMA * 1.02 * np.sqrt(np.maximum(var_dz, 0.0)) + np.abs(slack) + 1e-5 * np.abs(np.take_along_axis(dz_o, ids.astype(np.int64), axis=1)) + 1e-30
    err = np.abs(np.take_along_axis(dz - dz_o, ids.astype(np.int64), axis=1))
    worst = float((err / bound).max())
    say(f"  R={R} dX rms {ex[0]:.5f} max {ex[1]:.5f}; weight gradients rms {ew[0]:.5f} max {ew[1]:.5f}; dlogits rms {rel:.5f}, "
        f"largest entry error / storage-format bound {worst:.3f}")
    assert rel <= BWD_RMS_TOL
    assert worst <= 1.0
    assert np.array_equal(dz != 0, dz_o != 0) or np.abs(dz - dz_o)[(dz != 0) != (dz_o != 0)].max() < 1e-12
    p.wl.drop_weights()
    torch.cuda.empty_cache()


def test_grouped_ffn_backward_over_random_shapes():
    # random group counts and sizes (empty groups, single rows, sizes around the 32-row window and
    # the 256-row tile), random widths: every case against the oracle
    rng = np.random.default_rng(2024)
    pool = [0, 0, 1, 2, 31, 32, 33, 63, 64, 65, 100, 255, 256, 257, 300, 511, 513]
    for case in range(8):
        G = int(rng.integers(1, 9))
        sizes = [int(rng.choice(pool)) for _ in range(G)]
        d = int(rng.choice([256, 512, 768]))
        f = int(rng.choice([256, 512]))
        say(f"ffn backward random case {case}: sizes={sizes} d={d} f={f}")
        r = run_forward_backward(sizes, d, f, torch.float32, pad=int(rng.integers(0, 40)), seed=100 + case)
        (dXp_o, grads_o), _ = oracle_backward(r)
        if r["R"]:
            check_rows(f64(r["dXp"])[:r["R"]], dXp_o, f"case {case}: dXp")
        check_weight_grads(r, grads_o, f"case {case}")
        assert (r["dXp"][r["R"]:].float() == 512.0).all()


def test_weight_gradients_accumulate_over_micro_batches():
    # two micro-batches into the same fp32 gradient buffers: overwrite, then accumulate; the sum
    # against the oracle's two gradients, and an empty group's buffers left as they were
    d, f = 256, 256
    batches = [[70, 0, 300], [33, 5, 0]]
    G = 3
    W = make_weights(G, d, f, 31)
    Wd = [tuple(m.to(DEV) for m in w) for w in W]
    wl = [[w[i] for w in Wd] for i in range(3)]
    Wo = [tuple(f64(m) for m in w) for w in W]
    dW = [[torch.full(s, 5.0, dtype=torch.float32, device=DEV) for _ in range(G)] for s in ((d, f), (d, f), (f, d))]
    want = [[np.zeros(s) for s in ((d, f), (d, f), (f, d))] for _ in range(G)]
    for bi, sizes in enumerate(batches):
        off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        R = int(off[-1])
        gen = torch.Generator().manual_seed(40 + bi)
        Xp = torch.randn((R, d), generator=gen).to(torch.bfloat16)
        dYp = torch.randn((R, d), generator=gen).to(torch.bfloat16)
        H = torch.zeros((R, f), dtype=torch.bfloat16, device=DEV)
        AB = torch.zeros((R, 2 * f), dtype=torch.bfloat16, device=DEV)
        Yp = torch.zeros((R, d), dtype=torch.float32, device=DEV)
        dXp = torch.zeros((R, d), dtype=torch.float32, device=DEV)
        off_dev = torch.from_numpy(off).to(DEV)
        fe.feplb_grouped_ffn(Xp.to(DEV), off_dev, 0, G, d, f, *wl, H, Yp, AB=AB)
        B.feplb_grouped_ffn_backward(Xp.to(DEV), off_dev, 0, G, d, f, *wl, H, AB, dYp.to(DEV), dXp, *dW,
                                     phases=B.BWD_ALL | (B.BWD_ACCUMULATE if bi else 0))
        torch.cuda.synchronize()
        _, grads = orc.grouped_ffn_backward(f64(Xp), off, Wo, f64(dYp))
        for g in range(G):
            for i in range(3):
                want[g][i] += grads[g][i]
    for g in range(G):
        for i in range(3):
            check_rows(f64(dW[i][g]), want[g][i], f"accumulated gradient {i} of group {g}")
    # group 1 was empty in the first batch (zeros written) and had 5 rows in the second
    # a group that is empty in an accumulating call keeps its contents bit for bit
    before = [m.clone() for m in (dW[0][2], dW[1][2], dW[2][2])]
    off = torch.tensor([0, 40, 40, 40], dtype=torch.int32, device=DEV)
    z = torch.randn((40, d), generator=torch.Generator().manual_seed(9)).to(torch.bfloat16).to(DEV)
    H = torch.zeros((40, f), dtype=torch.bfloat16, device=DEV)
    AB = torch.zeros((40, 2 * f), dtype=torch.bfloat16, device=DEV)
    Yp = torch.zeros((40, d), dtype=torch.float32, device=DEV)
    dXp = torch.zeros((40, d), dtype=torch.float32, device=DEV)
    fe.feplb_grouped_ffn(z, off, 0, G, d, f, *wl, H, Yp, AB=AB)
    B.feplb_grouped_ffn_backward(z, off, 0, G, d, f, *wl, H, AB, z, dXp, *dW, phases=B.BWD_ALL | B.BWD_ACCUMULATE)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(before, (dW[0][2], dW[1][2], dW[2][2])))


def test_backward_capacity_below_the_row_count_truncates():
    # offsets promise more rows than the buffers hold: every kernel stops at R_cap
    d, f = 256, 256
    sizes = [100, 60, 80]
    R_cap = 130                      # group 1 is cut to 30 rows, group 2 to none
    off_full = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    off_cut = np.minimum(off_full, R_cap).astype(np.int32)
    gen = torch.Generator().manual_seed(77)
    Xp = torch.randn((R_cap, d), generator=gen).to(torch.bfloat16)
    dYp = torch.randn((R_cap, d), generator=gen).to(torch.bfloat16)
    W = make_weights(3, d, f, 78)
    Wd = [tuple(m.to(DEV) for m in w) for w in W]
    wl = [[w[i] for w in Wd] for i in range(3)]
    H = torch.zeros((R_cap, f), dtype=torch.bfloat16, device=DEV)
    AB = torch.zeros((R_cap, 2 * f), dtype=torch.bfloat16, device=DEV)
    Yp = torch.zeros((R_cap, d), dtype=torch.float32, device=DEV)
    dXp = torch.zeros((R_cap, d), dtype=torch.float32, device=DEV)
    dW = [[torch.full(s, 2.0, dtype=torch.float32, device=DEV) for _ in range(3)] for s in ((d, f), (d, f), (f, d))]
    off_dev = torch.from_numpy(off_full).to(DEV)
    fe.feplb_grouped_ffn(Xp.to(DEV), off_dev, 0, 3, d, f, *wl, H, Yp, AB=AB)
    B.feplb_grouped_ffn_backward(Xp.to(DEV), off_dev, 0, 3, d, f, *wl, H, AB, dYp.to(DEV), dXp, *dW)
    torch.cuda.synchronize()
    Wo = [tuple(f64(m) for m in w) for w in W]
    dXp_o, grads_o = orc.grouped_ffn_backward(f64(Xp), off_cut, Wo, f64(dYp))
    check_rows(f64(dXp), dXp_o, "dXp")
    r = dict(offsets=off_cut, dW=list(zip(*dW)))
    check_weight_grads(r, grads_o, "truncated")


def test_training_step_with_the_largest_group_count():
    # 128 groups (the limit of the by-value pointer tables), most of them tiny or empty
    rng = np.random.default_rng(128)
    sizes = [int(v) for v in rng.choice([0, 0, 1, 3, 17, 40, 70], size=B.MAX_GROUPS)]
    sizes[5], sizes[77], sizes[127] = 300, 260, 33
    d, f = 256, 256
    say(f"ffn backward with {len(sizes)} groups, {sum(sizes)} rows")
    r = run_forward_backward(sizes, d, f, torch.float32, seed=128)
    (dXp_o, grads_o), _ = oracle_backward(r)
    check_rows(f64(r["dXp"])[:r["R"]], dXp_o, "dXp")
    check_weight_grads(r, grads_o, "128 groups")
    # the forward's outputs on the same call: Yp against the oracle
    _, Yp_o = orc.grouped_ffn(f64(r["Xp"])[:r["R"]], r["offsets"], [tuple(f64(m) for m in w) for w in r["W"]])
    assert row_rel_err(f64(r["Yp"])[:r["R"]], Yp_o).max() <= 2e-2
    with pytest.raises(B.FeplbError):       # one group more than the tables hold
        off = torch.zeros((B.MAX_GROUPS + 2,), dtype=torch.int32, device=DEV)
        z = torch.zeros((64, d), dtype=torch.bfloat16, device=DEV)
        w = [torch.zeros((d, f), dtype=torch.bfloat16, device=DEV)] * (B.MAX_GROUPS + 1)
        fe.feplb_grouped_ffn(z, off, 0, B.MAX_GROUPS + 1, d, f, w, w, w, torch.zeros((64, f), dtype=torch.bfloat16, device=DEV),
                             torch.zeros((64, d), dtype=torch.float32, device=DEV))


def test_training_forward_gathering_rows_equals_reading_the_permuted_copy():
    # feplb_grouped_ffn_train with row_src (rows gathered from X as they are loaded) against the
    # same call on a materialised Xp: H, the kept derivatives and Yp bit for bit
    T, E, k, d, f = 700, 8, 2, 512, 256
    rng = np.random.default_rng(5)
    ids = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    groups = [(e, 0, B.ORD_MAX) for e in (0, 3, 5, 6)]
    G = len(groups)
    X = torch.randn((T, d), generator=torch.Generator().manual_seed(6)).to(torch.bfloat16).to(DEV)
    R_cap = T * k
    Xp, offsets, row_src, inv = B.feplb_permute(torch.from_numpy(ids).to(DEV), E, groups, X, R_cap)
    W = [tuple(m.to(DEV) for m in w) for w in make_weights(G, d, f, 9)]
    wl = [[w[i] for w in W] for i in range(3)]
    outs = []
    for gather in (False, True):
        H = torch.zeros((R_cap, f), dtype=torch.bfloat16, device=DEV)
        AB = torch.zeros((R_cap, 2 * f), dtype=torch.bfloat16, device=DEV)
        Yp = torch.zeros((R_cap, d), dtype=torch.float32, device=DEV)
        if gather:
            fe.feplb_grouped_ffn(X, offsets, 0, G, d, f, *wl, H, Yp, AB=AB, row_src=row_src, k=k)
        else:
            fe.feplb_grouped_ffn(Xp, offsets, 0, G, d, f, *wl, H, Yp, AB=AB)
        torch.cuda.synchronize()
        outs.append((H, AB, Yp))
    assert all(torch.equal(a, b) for a, b in zip(*outs))
    # and the plain forward writes the same H and Yp as the training forward
    H = torch.zeros((R_cap, f), dtype=torch.bfloat16, device=DEV)
    Yp = torch.zeros((R_cap, d), dtype=torch.float32, device=DEV)
    fe.feplb_grouped_ffn(Xp, offsets, 0, G, d, f, *wl, H, Yp)
    torch.cuda.synchronize()
    assert torch.equal(H, outs[0][0]) and torch.equal(Yp, outs[0][2])
