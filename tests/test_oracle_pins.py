"""Pins for the CPU oracle: each function is checked against something other
than itself -- values the paper prints, closed forms, brute force written with
scalar Python loops, library routines on special cases, and invariants --
chosen so that a dropped term, a wrong sign or index, or a transposed operand
fails at least one test.  No GPU is needed."""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import feplb_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    moves = []
    with open(os.path.join(GOLD, name)) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, *vals = line.split()
            if key == "move":
                moves.append(tuple(int(v) for v in vals))
            else:
                out[key] = [float(v) if "." in v else int(v) for v in vals]
    out["moves"] = moves
    return out


# ---------------------------------------------------------------- routing
def brute_route(logits, k):
    """Scalar loops: repeated selection of the best remaining expert."""
    T, E = logits.shape
    ids = np.zeros((T, k), dtype=np.int32)
    w = np.zeros((T, k))
    for t in range(T):
        row = [float(v) for v in logits[t]]
        m = max(row)
        ex = [math.exp(v - m) for v in row]
        s = sum(ex)
        p = [v / s for v in ex]
        taken = []
        for j in range(k):
            best = -1
            for e in range(E):
                if e in taken:
                    continue
                if best < 0 or row[e] > row[best]:   # strict: lower id wins ties
                    best = e
            taken.append(best)
        tot = sum(p[e] for e in taken)
        for j, e in enumerate(taken):
            ids[t, j] = e
            w[t, j] = p[e] / tot
    return ids, w


def test_route_paper_style_closed_form():
    g = read_golden("route_example.txt")
    logits = np.log(np.array([g["p"]], dtype=np.float64)).astype(np.float32)
    ids, w, counts = orc.route_topk(logits, g["k"][0])
    assert ids.tolist() == [g["ids"]]
    want = np.array(g["w_num"]) / g["w_den"][0]
    assert np.allclose(w[0], want, atol=1e-7)   # logits were rounded to fp32
    assert counts.tolist() == [0, 0, 1, 1]


@pytest.mark.parametrize("T,E,k,seed", [(37, 8, 2, 0), (16, 128, 8, 1), (5, 5, 5, 2), (9, 3, 1, 3)])
def test_route_matches_brute_force(T, E, k, seed):
    rng = np.random.default_rng(seed)
    logits = rng.normal(size=(T, E)).astype(np.float32)
    ids, w, counts = orc.route_topk(logits, k)
    bids, bw = brute_route(logits, k)
    assert np.array_equal(ids, bids)
    assert np.allclose(w, bw, rtol=0, atol=1e-14)
    assert counts.sum() == T * k
    assert np.array_equal(counts, np.bincount(bids.ravel(), minlength=E))


def test_route_k_equals_E_is_softmax():
    rng = np.random.default_rng(5)
    logits = rng.normal(size=(11, 16)).astype(np.float32)
    ids, w, _ = orc.route_topk(logits, 16)
    sm = scipy.special.softmax(logits.astype(np.float64), axis=1)
    assert np.allclose(w, np.take_along_axis(sm, ids.astype(np.int64), 1), atol=1e-14)
    assert np.all(np.sort(ids, axis=1) == np.arange(16))


def test_route_invariants_and_order():
    rng = np.random.default_rng(6)
    logits = (rng.normal(size=(200, 128)) - 2.4 * np.log(rng.permutation(128) + 1)).astype(np.float32)
    ids, w, counts = orc.route_topk(logits, 8)
    assert ids.min() >= 0 and ids.max() < 128
    assert all(len(set(r)) == 8 for r in ids.tolist())
    assert np.all(np.diff(w, axis=1) <= 0)              # position 0 holds the largest
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-14)
    assert counts.sum() == 200 * 8
    # the kept logits are the 8 largest of the row
    kept = np.take_along_axis(logits, ids.astype(np.int64), 1)
    assert np.array_equal(kept, -np.sort(-logits, axis=1)[:, :8])
    # equivalently: a softmax over the k kept logits alone
    assert np.allclose(w, scipy.special.softmax(kept.astype(np.float64), axis=1), atol=1e-14)


def test_route_ties_and_signed_zero_and_shift():
    logits = np.array([[1.0, 3.0, 3.0, 1.0, 3.0],
                       [0.0, -0.0, 0.0, -0.0, -1.0]], dtype=np.float32)
    ids, w, _ = orc.route_topk(logits, 3)
    assert ids.tolist() == [[1, 2, 4], [0, 1, 2]]
    assert np.allclose(w, 1.0 / 3.0)
    ids2, w2, _ = orc.route_topk(logits + np.float32(8.0), 3)
    assert np.array_equal(ids, ids2) and np.allclose(w, w2, atol=1e-12)
    big = np.full((1, 6), -30.0, dtype=np.float32)
    big[0, 4] = 30.0
    ids3, w3, _ = orc.route_topk(big, 2)
    assert ids3[0, 0] == 4 and ids3[0, 1] == 0 and abs(w3[0, 0] - 1.0) < 1e-20 + 1e-12


def test_route_rejects_bad_arguments():
    with pytest.raises(ValueError):
        orc.route_topk(np.zeros((2, 4), np.float32), 5)
    with pytest.raises(ValueError):
        orc.route_topk(np.array([[np.nan, 0.0]], np.float32), 1)


# ---------------------------------------------------------------- permutation
def brute_permute(ids, groups):
    """O(A^2 + A*G) counting definition: ordinal of a = number of earlier
    assignments with the same expert; row = group start + number of earlier
    members of the same group."""
    flat = [int(v) for v in np.asarray(ids).reshape(-1)]
    A = len(flat)
    grp = [-1] * A
    for a in range(A):
        o = sum(1 for b in range(a) if flat[b] == flat[a])
        for g, (e, lo, hi) in enumerate(groups):
            if e == flat[a] and lo <= o < hi:
                grp[a] = g
    G = len(groups)
    sizes = [sum(1 for a in range(A) if grp[a] == g) for g in range(G)]
    offsets = [0]
    for s in sizes:
        offsets.append(offsets[-1] + s)
    inv = [-1] * A
    for a in range(A):
        if grp[a] >= 0:
            inv[a] = offsets[grp[a]] + sum(1 for b in range(a) if grp[b] == grp[a])
    row_src = [0] * offsets[-1]
    for a in range(A):
        if inv[a] >= 0:
            row_src[inv[a]] = a
    return offsets, row_src, inv


def check_permutation_invariants(ids, groups, offsets, row_src, inv):
    flat = np.asarray(ids).reshape(-1)
    R = int(offsets[-1])
    assert offsets[0] == 0 and np.all(np.diff(offsets) >= 0)
    assert row_src.shape[0] == R
    assert np.array_equal(inv[row_src], np.arange(R))           # bijection rows <-> kept assignments
    assert int((inv >= 0).sum()) == R
    for g, (e, lo, hi) in enumerate(groups):
        seg = row_src[offsets[g]:offsets[g + 1]]
        assert np.all(np.diff(seg) > 0)                         # stable inside a group
        assert np.all(flat[seg] == e)
        occ = np.nonzero(flat == e)[0]
        assert np.array_equal(seg, occ[lo:hi])                  # exactly occurrences lo..hi-1


def test_permute_hand_example():
    # 3 tokens, top-2; experts per slot: t0:(2,0) t1:(0,2) t2:(2,1)
    ids = np.array([[2, 0], [0, 2], [2, 1]], dtype=np.int32)
    # groups: expert 0 (all), expert 2 occurrences [0,2), expert 2 occurrences [2,inf); expert 1 is not local
    groups = [(0, 0, orc.INT32_MAX), (2, 0, 2), (2, 2, orc.INT32_MAX)]
    offsets, row_src, inv = orc.permute(ids, groups)
    assert offsets.tolist() == [0, 2, 4, 5]
    assert row_src.tolist() == [1, 2, 0, 3, 4]
    assert inv.tolist() == [2, 0, 1, 3, 4, -1]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_permute_matches_brute_force(seed):
    rng = np.random.default_rng(seed)
    T, E, k = 23, 6, 3
    logits = rng.normal(size=(T, E)).astype(np.float32)
    ids, _, counts = orc.route_topk(logits, k)
    n4 = int(counts[4])
    groups = [(1, 0, orc.INT32_MAX), (4, n4 // 2, orc.INT32_MAX), (0, 0, orc.INT32_MAX),
              (4, 0, n4 // 2), (5, 2, 5), (3, 10**6, orc.INT32_MAX)]
    offsets, row_src, inv = orc.permute(ids, groups)
    bo, br, bi = brute_permute(ids, groups)
    assert offsets.tolist() == bo and row_src.tolist() == br and inv.tolist() == bi
    check_permutation_invariants(ids, groups, offsets, row_src, inv)


def test_permute_all_local_keeps_every_assignment():
    rng = np.random.default_rng(3)
    T, E, k = 64, 8, 2
    ids, _, counts = orc.route_topk(rng.normal(size=(T, E)).astype(np.float32), k)
    groups = [(e, 0, orc.INT32_MAX) for e in range(E)]
    offsets, row_src, inv = orc.permute(ids, groups)
    assert offsets[-1] == T * k
    assert np.array_equal(np.diff(offsets), counts)
    check_permutation_invariants(ids, groups, offsets, row_src, inv)
    X = rng.normal(size=(T, 5))
    Xp = orc.gather_rows(X, row_src, k)
    for r in range(T * k):
        assert np.array_equal(Xp[r], X[row_src[r] // k])


def test_permute_empty_inputs():
    offsets, row_src, inv = orc.permute(np.zeros((0, 2), np.int32), [(0, 0, 5)])
    assert offsets.tolist() == [0, 0] and row_src.size == 0 and inv.size == 0
    offsets, row_src, inv = orc.permute(np.array([[0, 1]], np.int32), [])
    assert offsets.tolist() == [0] and inv.tolist() == [-1, -1]


# ---------------------------------------------------------------- expert FFN
def silu(z):
    return z / (1.0 + math.exp(-z))


def brute_ffn(x, wg, wu, wd):
    m, d = x.shape
    f = wg.shape[1]
    h = [[0.0] * f for _ in range(m)]
    y = [[0.0] * d for _ in range(m)]
    for r in range(m):
        for j in range(f):
            a = sum(float(x[r, i]) * float(wg[i, j]) for i in range(d))
            b = sum(float(x[r, i]) * float(wu[i, j]) for i in range(d))
            h[r][j] = silu(a) * b
        for i in range(d):
            y[r][i] = sum(h[r][j] * float(wd[j, i]) for j in range(f))
    return np.array(h), np.array(y)


def test_ffn_matches_scalar_loops():
    rng = np.random.default_rng(0)
    m, d, f = 5, 7, 9                      # d != f so a transposed operand cannot even multiply
    x = rng.normal(size=(m, d))
    wg, wu, wd = rng.normal(size=(d, f)), rng.normal(size=(d, f)), rng.normal(size=(f, d))
    h, y = orc.ffn_rows(x, wg, wu, wd)
    bh, by = brute_ffn(x, wg, wu, wd)
    assert np.allclose(h, bh, rtol=1e-12, atol=1e-12)
    assert np.allclose(y, by, rtol=1e-12, atol=1e-12)


def test_ffn_single_entry_weights_closed_form():
    # square shapes would hide a transposed operand; single non-symmetric entries expose it
    d = f = 4
    x = np.array([[0.5, -1.0, 2.0, 3.0]])
    wg = np.zeros((d, f)); wg[0, 1] = 1.0     # a_1 = x_0
    wu = np.zeros((d, f)); wu[2, 1] = 1.0     # b_1 = x_2
    wd = np.zeros((f, d)); wd[1, 3] = 1.0     # y_3 = h_1
    h, y = orc.ffn_rows(x, wg, wu, wd)
    want = silu(0.5) * 2.0
    assert np.allclose(h, [[0, want, 0, 0]], atol=1e-15)
    assert np.allclose(y, [[0, 0, 0, want]], atol=1e-15)
    # gate and up are not interchangeable: silu acts on the gate only
    h2, _ = orc.ffn_rows(x, wu, wg, wd)
    assert np.allclose(h2[0, 1], silu(2.0) * 0.5, atol=1e-15)
    assert abs(h2[0, 1] - want) > 0.1


def test_ffn_activation_limits():
    d = f = 3
    eye = np.eye(3)
    x = np.array([[0.0, 40.0, -40.0]])
    h, _ = orc.ffn_rows(x, eye, eye, eye)
    # silu(0) = 0; silu(z) -> z for large z; silu(z) -> 0 for very negative z
    assert h[0, 0] == 0.0
    assert abs(h[0, 1] - 1600.0) < 1e-9
    assert abs(h[0, 2]) < 1e-12


def test_ffn_torch_library_special_case():
    rng = np.random.default_rng(1)
    m, d, f = 33, 48, 20
    x, wg, wu, wd = (rng.normal(size=s) for s in ((m, d), (d, f), (d, f), (f, d)))
    h, y = orc.ffn_rows(x, wg, wu, wd)
    tx, tg, tu, td = (torch.from_numpy(v) for v in (x, wg, wu, wd))
    th = torch.nn.functional.silu(tx @ tg) * (tx @ tu)
    assert np.allclose(h, th.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(y, (th @ td).numpy(), rtol=1e-11, atol=1e-11)


def test_ffn_linearity_and_row_independence():
    rng = np.random.default_rng(2)
    m, d, f = 6, 8, 5
    x, wg, wu, wd, wd2 = (rng.normal(size=s) for s in ((m, d), (d, f), (d, f), (f, d), (f, d)))
    _, y1 = orc.ffn_rows(x, wg, wu, wd)
    _, y2 = orc.ffn_rows(x, wg, wu, wd2)
    _, y12 = orc.ffn_rows(x, wg, wu, 2.0 * wd - 3.0 * wd2)
    assert np.allclose(y12, 2.0 * y1 - 3.0 * y2, atol=1e-11)
    perm = rng.permutation(m)
    _, yp = orc.ffn_rows(x[perm], wg, wu, wd)
    assert np.allclose(yp, y1[perm], atol=1e-12)


def test_grouped_ffn_uses_each_groups_own_weights_and_skips_empty():
    rng = np.random.default_rng(3)
    d, f = 6, 4
    offsets = np.array([0, 3, 3, 7], dtype=np.int32)          # middle group empty
    Xp = rng.normal(size=(7, d))
    ws = [tuple(rng.normal(size=s) for s in ((d, f), (d, f), (f, d))) for _ in range(3)]
    H, Yp = orc.grouped_ffn(Xp, offsets, ws)
    for g, (lo, hi) in enumerate([(0, 3), (3, 3), (3, 7)]):
        if hi > lo:
            bh, by = brute_ffn(Xp[lo:hi], *ws[g])
            assert np.allclose(H[lo:hi], bh, atol=1e-12) and np.allclose(Yp[lo:hi], by, atol=1e-12)


# ---------------------------------------------------------------- expert FFN, backward
def test_ffn_backward_matches_central_differences_of_the_forward():
    # the gradient of L = sum(y * dy) with respect to every input, from the forward definition alone
    rng = np.random.default_rng(10)
    m, d, f = 3, 5, 4                      # d != f so a transposed operand cannot even multiply
    x, wg, wu, wd, dy = (rng.normal(size=s) for s in ((m, d), (d, f), (d, f), (f, d), (m, d)))
    got = orc.ffn_rows_backward(x, wg, wu, wd, dy)

    def loss(x_, wg_, wu_, wd_):
        return float(np.sum(orc.ffn_rows(x_, wg_, wu_, wd_)[1] * dy))

    args = [x, wg, wu, wd]
    eps = 1e-5
    for which in range(4):
        num = np.zeros_like(args[which])
        for idx in np.ndindex(*args[which].shape):
            hi = [a.copy() for a in args]
            lo = [a.copy() for a in args]
            hi[which][idx] += eps
            lo[which][idx] -= eps
            num[idx] = (loss(*hi) - loss(*lo)) / (2 * eps)
        assert np.allclose(got[which], num, rtol=1e-7, atol=1e-8), which


def test_ffn_backward_torch_autograd_special_case():
    rng = np.random.default_rng(11)
    m, d, f = 17, 24, 10
    x, wg, wu, wd, dy = (rng.normal(size=s) for s in ((m, d), (d, f), (d, f), (f, d), (m, d)))
    tx, tg, tu, td = (torch.from_numpy(v).requires_grad_(True) for v in (x, wg, wu, wd))
    y = (torch.nn.functional.silu(tx @ tg) * (tx @ tu)) @ td
    y.backward(torch.from_numpy(dy))
    got = orc.ffn_rows_backward(x, wg, wu, wd, dy)
    for g, t in zip(got, (tx, tg, tu, td)):
        assert np.allclose(g, t.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_ffn_backward_single_entry_closed_form():
    # one path through the expert: y_3 = silu(x_0) * x_2, so every gradient is a scalar formula
    d = f = 4
    x = np.array([[0.5, -1.0, 2.0, 3.0]])
    wg = np.zeros((d, f)); wg[0, 1] = 1.0
    wu = np.zeros((d, f)); wu[2, 1] = 1.0
    wd = np.zeros((f, d)); wd[1, 3] = 1.0
    dy = np.array([[7.0, 0.0, 0.0, 1.5]])          # only dy_3 can matter
    a, b = 0.5, 2.0
    sg = 1.0 / (1.0 + math.exp(-a))
    dsilu = sg * (1.0 + a * (1.0 - sg))
    dx, dwg, dwu, dwd = orc.ffn_rows_backward(x, wg, wu, wd, dy)
    want_dx = np.zeros((1, d)); want_dx[0, 0] = 1.5 * b * dsilu; want_dx[0, 2] = 1.5 * silu(a)
    assert np.allclose(dx, want_dx, atol=1e-15)
    # dWg[i,1] = x_i * da_1, dWu[i,1] = x_i * db_1, dWd[1,i] = h_1 * dy_i; everything else zero
    want = np.zeros((d, f)); want[:, 1] = x[0] * (1.5 * b * dsilu)
    assert np.allclose(dwg, want, atol=1e-15)
    want = np.zeros((d, f)); want[:, 1] = x[0] * (1.5 * silu(a))
    assert np.allclose(dwu, want, atol=1e-15)
    want = np.zeros((f, d)); want[1, :] = silu(a) * b * dy[0]
    assert np.allclose(dwd, want, atol=1e-15)


def test_ffn_backward_is_linear_in_dy_and_sums_weight_gradients_over_rows():
    rng = np.random.default_rng(12)
    m, d, f = 6, 8, 5
    x, wg, wu, wd, dy1, dy2 = (rng.normal(size=s) for s in ((m, d), (d, f), (d, f), (f, d), (m, d), (m, d)))
    g1 = orc.ffn_rows_backward(x, wg, wu, wd, dy1)
    g2 = orc.ffn_rows_backward(x, wg, wu, wd, dy2)
    g12 = orc.ffn_rows_backward(x, wg, wu, wd, 2.0 * dy1 - 3.0 * dy2)
    for a, b, c in zip(g1, g2, g12):
        assert np.allclose(c, 2.0 * a - 3.0 * b, atol=1e-11)
    # rows are independent: dx row by row, weight gradients are the sum over the rows
    parts = [orc.ffn_rows_backward(x[r:r + 1], wg, wu, wd, dy1[r:r + 1]) for r in range(m)]
    assert np.allclose(np.concatenate([p_[0] for p_ in parts]), g1[0], atol=1e-12)
    for i in (1, 2, 3):
        assert np.allclose(sum(p_[i] for p_ in parts), g1[i], atol=1e-11)
    assert all(np.all(v == 0) for v in orc.ffn_rows_backward(x, wg, wu, wd, np.zeros((m, d))))


def test_grouped_ffn_backward_uses_each_groups_own_rows_and_weights():
    rng = np.random.default_rng(13)
    d, f = 6, 4
    offsets = np.array([0, 3, 3, 7], dtype=np.int32)          # middle group empty
    Xp, dYp = rng.normal(size=(7, d)), rng.normal(size=(7, d))
    ws = [tuple(rng.normal(size=s) for s in ((d, f), (d, f), (f, d))) for _ in range(3)]
    dXp, grads = orc.grouped_ffn_backward(Xp, offsets, ws, dYp)
    for g, (lo, hi) in enumerate([(0, 3), (3, 3), (3, 7)]):
        if hi > lo:
            want = orc.ffn_rows_backward(Xp[lo:hi], *ws[g], dYp[lo:hi])
            assert np.array_equal(dXp[lo:hi], want[0])
            assert all(np.array_equal(a, b) for a, b in zip(grads[g], want[1:]))
        else:
            assert all(np.all(v == 0) for v in grads[g])
            assert [v.shape for v in grads[g]] == [(d, f), (d, f), (f, d)]
    # the whole-batch loss differentiated numerically through grouped_ffn, a few coordinates
    def loss(Xq, wsq):
        return float(np.sum(orc.grouped_ffn(Xq, offsets, wsq)[1] * dYp))
    eps = 1e-5
    for (r, c) in [(0, 0), (4, 5), (6, 2)]:
        hi_, lo_ = Xp.copy(), Xp.copy()
        hi_[r, c] += eps; lo_[r, c] -= eps
        assert abs((loss(hi_, ws) - loss(lo_, ws)) / (2 * eps) - dXp[r, c]) < 1e-7
    for (g, which, idx) in [(0, 0, (1, 2)), (2, 1, (5, 3)), (2, 2, (3, 4)), (1, 0, (0, 0))]:
        hi_ = [list(w) for w in ws]; lo_ = [list(w) for w in ws]
        hi_[g][which] = hi_[g][which].copy(); lo_[g][which] = lo_[g][which].copy()
        hi_[g][which][idx] += eps; lo_[g][which][idx] -= eps
        num = (loss(Xp, hi_) - loss(Xp, lo_)) / (2 * eps)
        assert abs(num - grads[g][which][idx]) < 1e-7


# ---------------------------------------------------------------- layer backward: combine, permute, router
def test_combine_backward_matches_central_differences_and_scalar_loops():
    rng = np.random.default_rng(20)
    T, k, d, R = 6, 3, 5, 9
    inv = np.full(T * k, -1, dtype=np.int32)
    slots = rng.permutation(T * k)[:R]
    inv[slots] = rng.permutation(R)               # a bijection between R slots and R rows
    Yp, dY, w = rng.normal(size=(R, d)), rng.normal(size=(T, d)), rng.uniform(0.1, 1.0, size=(T, k))
    dYp, dw = orc.combine_backward(dY, Yp, inv, w, T, k)
    # scalar loops straight from the definition
    for t in range(T):
        for j in range(k):
            r = inv[t * k + j]
            if r >= 0:
                assert np.allclose(dYp[r], w[t, j] * dY[t], atol=1e-14)
                assert abs(dw[t, j] - sum(dY[t, i] * Yp[r, i] for i in range(d))) < 1e-12
            else:
                assert dw[t, j] == 0.0
    # central differences of L = sum(combine(...) * dY)
    def loss(Yp_, w_):
        return float(np.sum(orc.combine(Yp_, inv, w_, T, k) * dY))
    eps = 1e-6
    for idx in [(0, 0), (4, 2), (8, 4)]:
        hi, lo = Yp.copy(), Yp.copy()
        hi[idx] += eps; lo[idx] -= eps
        assert abs((loss(hi, w) - loss(lo, w)) / (2 * eps) - dYp[idx]) < 1e-8
    for t in range(T):
        for j in range(k):
            hi, lo = w.copy(), w.copy()
            hi[t, j] += eps; lo[t, j] -= eps
            assert abs((loss(Yp, hi) - loss(Yp, lo)) / (2 * eps) - dw[t, j]) < 1e-8


def test_permute_backward_sums_the_copies_of_a_token():
    rng = np.random.default_rng(21)
    T, E, k, d = 12, 6, 3, 4
    ids = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    groups = [(0, 0, orc.INT32_MAX), (3, 0, orc.INT32_MAX), (5, 0, 2), (5, 2, orc.INT32_MAX)]
    offsets, row_src, inv = orc.permute(ids, groups)
    R = int(offsets[-1])
    dXp = rng.normal(size=(R, d))
    dX = orc.permute_backward(dXp, inv, T, k)
    want = np.zeros((T, d))
    for r in range(R):
        want[row_src[r] // k] += dXp[r]
    assert np.allclose(dX, want, atol=1e-14)
    # adjoint of the gather: <gather(X), dXp> = <X, dX>
    X = rng.normal(size=(T, d))
    assert abs(np.sum(orc.gather_rows(X, row_src, k) * dXp) - np.sum(X * dX)) < 1e-12


def test_route_backward_matches_central_differences_and_torch():
    rng = np.random.default_rng(22)
    T, E, k = 7, 9, 4
    z = rng.normal(size=(T, E)).astype(np.float32)
    ids, w, _ = orc.route_topk(z, k)
    dw = rng.normal(size=(T, k))
    dz = orc.route_topk_backward(z, ids, dw)
    eps = 1e-3                                           # fp32 logits: a step the selection survives
    z64 = z.astype(np.float64)
    def weights_at(zz):
        kept = np.take_along_axis(zz, ids.astype(np.int64), axis=1)
        p = np.exp(zz - zz.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        pk = np.take_along_axis(p, ids.astype(np.int64), axis=1)
        return pk / pk.sum(axis=1, keepdims=True)
    assert np.allclose(weights_at(z64), w, atol=1e-12)    # same function as the forward's weights
    for t, e in [(0, int(ids[0, 0])), (3, int(ids[3, 2])), (5, int(ids[5, 3])), (2, int(np.setdiff1d(np.arange(E), ids[2])[0]))]:
        hi, lo = z64.copy(), z64.copy()
        hi[t, e] += eps; lo[t, e] -= eps
        num = np.sum((weights_at(hi) - weights_at(lo)) * dw) / (2 * eps)
        assert abs(num - dz[t, e]) < 1e-6
    # torch: softmax over the kept logits
    tz = torch.from_numpy(z64).requires_grad_(True)
    tw = torch.softmax(torch.gather(tz, 1, torch.from_numpy(ids.astype(np.int64))), dim=1)
    tw.backward(torch.from_numpy(dw))
    assert np.allclose(dz, tz.grad.numpy(), atol=1e-12)
    # rows sum to zero (the weights sum to one), experts not kept get nothing
    assert np.abs(dz.sum(axis=1)).max() < 1e-12
    mask = np.ones((T, E), dtype=bool)
    np.put_along_axis(mask, ids.astype(np.int64), False, axis=1)
    assert not dz[mask].any()


# ---------------------------------------------------------------- combine, end to end
def small_layer(seed, T=40, E=8, k=2, d=12, f=10):
    rng = np.random.default_rng(seed)
    logits = rng.normal(size=(T, E)).astype(np.float32)
    X = rng.normal(size=(T, d))
    W = {e: tuple(0.3 * rng.normal(size=s) for s in ((d, f), (d, f), (f, d))) for e in range(E)}
    return logits, X, W


def run_oracle_layer(logits, X, W, k, groups):
    ids, w, counts = orc.route_topk(logits, k)
    offsets, row_src, inv = orc.permute(ids, groups)
    Xp = orc.gather_rows(X, row_src, k)
    _, Yp = orc.grouped_ffn(Xp, offsets, [W[e] for (e, _, _) in groups])
    return ids, w, counts, orc.combine(Yp, inv, w, X.shape[0], k)


def test_combine_matches_scalar_loops():
    rng = np.random.default_rng(0)
    T, k, d, R = 7, 3, 4, 9
    Yp = rng.normal(size=(R, d))
    inv = np.full(T * k, -1, dtype=np.int32)
    slots = rng.permutation(T * k)[:R]
    inv[slots] = np.arange(R)
    w = rng.uniform(size=(T, k))
    Y = orc.combine(Yp, inv, w, T, k)
    for t in range(T):
        for i in range(d):
            acc = 0.0
            for j in range(k):
                r = int(inv[t * k + j])
                if r >= 0:
                    acc += float(w[t, j]) * float(Yp[r, i])
            assert abs(Y[t, i] - acc) < 1e-14
    none = [t for t in range(T) if all(inv[t * k + j] < 0 for j in range(k))]
    for t in none:
        assert np.all(Y[t] == 0.0)


def test_layer_equals_per_token_definition_all_local():
    logits, X, W = small_layer(1)
    E, k = 8, 2
    groups = [(e, 0, orc.INT32_MAX) for e in range(E)]
    ids, w, _, Y = run_oracle_layer(logits, X, W, k, groups)
    for t in range(X.shape[0]):
        # scalar-loop FFN per slot, no permutation, no oracle FFN
        want = np.zeros(X.shape[1])
        for j in range(k):
            _, y = brute_ffn(X[t:t + 1], *W[int(ids[t, j])])
            want += w[t, j] * y[0]
        assert np.allclose(Y[t], want, atol=1e-12)
        assert np.allclose(Y[t], orc.moe_token(X[t], ids[t], w[t], W), atol=1e-12)


def test_layer_partial_locality_and_missing_tokens():
    logits, X, W = small_layer(2, T=60, E=16, k=3)
    local = [3, 4, 5, 9]
    groups = [(e, 0, orc.INT32_MAX) for e in local]
    ids, w, _, Y = run_oracle_layer(logits, X, W, 3, groups)
    Wl = {e: W[e] for e in local}
    seen_empty = False
    for t in range(60):
        want = orc.moe_token(X[t], ids[t], w[t], Wl)
        assert np.allclose(Y[t], want, atol=1e-12)
        if not any(int(e) in Wl for e in ids[t]):
            seen_empty = True
            assert np.all(Y[t] == 0.0)
    assert seen_empty


def test_batched_per_token_definition_matches_the_single_token_one():
    logits, X, W = small_layer(7, T=30, E=16, k=4)
    ids, w, _ = orc.route_topk(logits, 4)
    local = [1, 2, 8, 15]
    got = orc.moe_tokens(X, ids, w, np.isin(ids, local), lambda e: W[e])
    Wl = {e: W[e] for e in local}
    for t in range(30):
        assert np.allclose(got[t], orc.moe_token(X[t], ids[t], w[t], Wl), atol=1e-12)


def test_identical_experts_make_the_layer_a_plain_mlp():
    # with every expert equal, sum_j w_j FFN(x) = FFN(x) because the weights sum to one
    logits, X, W = small_layer(3)
    W = {e: W[0] for e in W}
    groups = [(e, 0, orc.INT32_MAX) for e in range(8)]
    _, _, _, Y = run_oracle_layer(logits, X, W, 2, groups)
    _, want = brute_ffn(X, *W[0])
    assert np.allclose(Y, want, atol=1e-12)


def test_output_does_not_depend_on_the_split_into_static_and_dynamic_groups():
    # Section 2.2: a token is processed by the same expert with the same weights wherever it runs
    logits, X, W = small_layer(4, T=80)
    k = 2
    ids, _, counts = orc.route_topk(logits, k)
    whole = [(e, 0, orc.INT32_MAX) for e in range(8)]
    n2, n5 = int(counts[2]), int(counts[5])
    split = [(e, 0, orc.INT32_MAX) for e in (0, 1, 3, 4, 6, 7)]
    split += [(2, 0, n2 // 3), (5, 0, n5 - 4), (5, n5 - 4, n5), (2, n2 // 3, n2)]
    Ya = run_oracle_layer(logits, X, W, k, whole)[3]
    Yb = run_oracle_layer(logits, X, W, k, split)[3]
    assert np.allclose(Ya, Yb, atol=1e-13)


# ---------------------------------------------------------------- plan
def test_paper_worked_numbers():
    g = {k: v[0] for k, v in read_golden("paper_worked_numbers.txt").items() if k != "moves"}
    E = g["experts_total"]
    assert orc.experts_per_device(E, 8) == g["ep8_experts_per_device"]
    assert orc.experts_per_device(E, 4) == g["ep4_experts_per_device"]
    assert orc.experts_per_device(E, 2) == g["ep2_experts_per_device"]
    assert orc.static_dynamic_split(E, 8, g["dyn"]) == (g["dyn4_static"], g["dyn4_dynamic"])
    assert orc.dynamic_buffer_bytes(1, g["d"], g["f"]) == g["expert_mib"] * 2**20
    assert orc.dynamic_buffer_bytes(g["max_num_dyn"], g["d"], g["f"]) == g["buffer_mib"] * 2**20


@pytest.mark.parametrize("name", ["plan_whole_example.txt", "plan_whole_tau_example.txt"])
def test_plan_whole_hand_worked(name):
    g = read_golden(name)
    moves, before, after = orc.plan_whole(g["P"][0], g["owner"], g["n"], g["dyn_flag"], g["slots"], g["tau"][0])
    assert before.tolist() == g["load_before"]
    assert after.tolist() == g["load_after"]
    assert [m[:4] for m in moves] == g["moves"]
    assert all(m[4] == 0 for m in moves)


def random_plan_case(rng, P, per):
    E = P * per
    owner = np.repeat(np.arange(P), per)
    n = (rng.pareto(1.2, size=E) * 50).astype(np.int64)
    n[rng.uniform(size=E) < 0.2] = 0
    dyn = (rng.uniform(size=E) < 0.5).astype(np.uint8)
    slots = rng.integers(0, 3, size=P)
    tau = int(rng.integers(0, 40))
    return E, owner, n, dyn, slots, tau


@pytest.mark.parametrize("seed", range(30))
def test_plan_whole_invariants(seed):
    rng = np.random.default_rng(seed)
    P, per = int(rng.integers(2, 9)), int(rng.integers(1, 17))
    E, owner, n, dyn, slots, tau = random_plan_case(rng, P, per)
    moves, before, after = orc.plan_whole(P, owner, n, dyn, slots, tau)
    assert before.sum() == after.sum() == n.sum()
    assert after.max() <= before.max()
    recv = np.zeros(P, dtype=int)
    seen = set()
    L = before.copy()
    for (e, src, dst, rows, lo) in moves:
        assert dyn[e] and n[e] >= max(tau, 1) and rows == n[e] and lo == 0
        assert src == owner[e] and dst != src and e not in seen
        assert L[dst] + rows < L[src] and L[src] == L.max()     # each step lowers the pair's maximum
        L[src] -= rows; L[dst] += rows
        seen.add(e); recv[dst] += 1
    assert np.array_equal(L, after)
    assert np.all(recv <= slots)
    assert orc.token_straggler(after) <= orc.token_straggler(before) + 1e-9
    again = orc.plan_whole(P, owner.copy(), n.copy(), dyn.copy(), slots.copy(), tau)
    assert again[0] == moves                                      # deterministic: every rank derives the same plan


def test_plan_whole_balanced_or_ineligible_means_no_moves():
    owner = np.repeat(np.arange(4), 2)
    n = np.full(8, 10)
    assert orc.plan_whole(4, owner, n, np.ones(8, np.uint8), [2] * 4, 1)[0] == []
    n = np.array([100, 90, 1, 1, 1, 1, 1, 1])
    assert orc.plan_whole(4, owner, n, np.zeros(8, np.uint8), [2] * 4, 1)[0] == []   # nothing dynamic
    assert orc.plan_whole(4, owner, n, np.ones(8, np.uint8), [0] * 4, 1)[0] == []    # no slots
    assert orc.plan_whole(4, owner, n, np.ones(8, np.uint8), [2] * 4, 101)[0] == []  # all below tau
    assert orc.plan_whole(4, owner, np.zeros(8, int), np.ones(8, np.uint8), [2] * 4, 0)[0] == []


def test_plan_whole_two_rank_closed_form():
    # P = 2, rank 0 holds experts a >= b, rank 1 is empty, plenty of slots:
    # the greedy moves a iff a < a + b (b > 0), then loads are (b, a); then rank 1 is the
    # most loaded but owns nothing, so it stops.
    for a, b in [(10, 3), (7, 7), (5, 0)]:
        moves, before, after = orc.plan_whole(2, [0, 0, 1], [a, b, 0], [1, 1, 1], [4, 4], 1)
        if b > 0:
            assert [m[:4] for m in moves] == [(0, 0, 1, a)] and after.tolist() == [b, a]
        else:
            assert moves == [] and after.tolist() == [a, 0]


@pytest.mark.parametrize("seed", range(12))
def test_plan_whole_against_exhaustive_search(seed):
    """Enumerate every placement of the dynamic experts (each stays or moves to
    another rank within the slot limits): the greedy result is never worse than
    doing nothing and never better than the best placement."""
    rng = np.random.default_rng(100 + seed)
    P, per = int(rng.integers(2, 4)), int(rng.integers(1, 4))
    E = P * per
    owner = np.repeat(np.arange(P), per)
    n = rng.integers(0, 30, size=E)
    dyn = np.ones(E, np.uint8)
    slots = rng.integers(0, 3, size=P)
    best = None
    for place in itertools.product(range(P), repeat=E):
        recv = [0] * P
        L = [0] * P
        for e, r in enumerate(place):
            L[r] += int(n[e])
            if r != owner[e]:
                recv[r] += 1
        if all(recv[r] <= slots[r] for r in range(P)):
            best = max(L) if best is None else min(best, max(L))
    moves, before, after = orc.plan_whole(P, owner, n, dyn, slots, 1)
    assert best <= after.max() <= before.max()


@pytest.mark.parametrize("seed", range(20))
def test_plan_overflow_invariants(seed):
    rng = np.random.default_rng(seed)
    P, per = int(rng.integers(2, 9)), int(rng.integers(2, 17))
    E, owner, n, dyn, slots, _ = random_plan_case(rng, P, per)
    this = orc.pick_receiver(P, owner, n)
    moves, before, after = orc.plan_overflow(P, owner, n, dyn, slots, this)
    M = -(-int(n.sum()) // P)
    assert before.sum() == after.sum() == n.sum()
    assert len(moves) <= slots[this]
    assert after[this] <= max(M, before[this])
    hot_n = sorted((int(n[e]) for e in range(E) if dyn[e] and owner[e] != this), reverse=True)[:len(moves)]
    assert sorted((int(n[m[0]]) for m in moves), reverse=True) == hot_n
    for (e, src, dst, rows, lo) in moves:
        assert dyn[e] and src == owner[e] != this and dst == this
        assert 0 <= rows <= n[e] and lo == n[e] - rows
    for r in range(P):
        if r != this:
            assert after[r] <= before[r]
    # receiver choice: brute force over ranks of |2L - M|
    d = [abs(2 * int(before[r]) - M) for r in range(P)]
    assert this == d.index(min(d))


def test_token_straggler_definition_and_paper_rows():
    assert orc.token_straggler([10, 20, 30, 40]) == 15.0
    assert orc.token_straggler([7, 7, 7]) == 0.0


# ---------------------------------------------------------------- macro level: placement from history
def test_history_update_fixed_point_average():
    n = np.array([0, 1, 7, 1000, 123456], dtype=np.int64)
    one = 1 << orc.HIST_FRAC_BITS
    # shift 0 keeps the last batch only, whatever the history was
    assert np.array_equal(orc.history_update(np.array([5, 0, 99, 1, 7]) * one, n, 0), n * one)
    # a constant count is a fixed point, approached monotonically from below and from above
    for start in (np.zeros(5, dtype=np.int64), 4 * n * one + 3):
        h = start.copy()
        for m in range(1, 200):
            h2 = orc.history_update(h, n, 3)
            assert np.all(np.abs(h2 - n * one) <= np.abs(h - n * one))
            h = h2
        assert np.all(np.abs(h - n * one) <= (1 << 3))            # within the flooring of the last steps
    assert np.array_equal(orc.history_update(n * one, n, 5), n * one)
    # against the real-valued recurrence h <- (1 - a) h + a n with a = 2^-shift: flooring loses < 1 unit per step
    rng = np.random.default_rng(0)
    h = np.zeros(5, dtype=np.int64)
    ref = np.zeros(5)
    for m in range(1, 40):
        c = rng.integers(0, 5000, size=5)
        h = orc.history_update(h, c, 2)
        ref = 0.75 * ref + 0.25 * (c * one)
        assert np.all(np.abs(h - ref) <= m)
    # the floor is towards minus infinity for a falling history too
    assert orc.history_update(np.array([10]), np.array([0]), 2)[0] == 10 + (-10 // 4) == 7


@pytest.mark.parametrize("name", ["place_lpt_graham_example.txt", "place_lpt_capacity_example.txt"])
def test_place_lpt_hand_worked(name):
    g = read_golden(name)
    owner, before, after, migrated = orc.place_lpt(g["P"][0], g["hist"], g["cap"][0], g["owner_in"])
    assert owner.tolist() == g["owner_out"]
    assert before.tolist() == g["load_before"] and after.tolist() == g["load_after"]
    assert migrated == g["migrated"][0]
    if "optimum" in g:
        m = g["P"][0]
        assert max(after) * 3 * m <= (4 * m - 1) * g["optimum"][0]           # Graham's bound, met with equality here
        assert max(after) * 3 * m == (4 * m - 1) * g["optimum"][0]


def best_makespan(P, hist, cap):
    """Exhaustive search over all maps with at most cap experts per rank."""
    best = None
    for assign in itertools.product(range(P), repeat=len(hist)):
        if max(np.bincount(assign, minlength=P)) > cap:
            continue
        load = np.bincount(assign, weights=hist, minlength=P).max()
        best = load if best is None else min(best, load)
    return best


@pytest.mark.parametrize("seed", range(12))
def test_place_lpt_against_exhaustive_search(seed):
    rng = np.random.default_rng(seed)
    P = int(rng.integers(2, 4))
    E = int(rng.integers(P, 8))
    hist = rng.integers(1, 50, size=E).astype(np.int64)
    everything_on_zero = np.zeros(E, dtype=np.int32)
    # without a binding limit this is Graham's list scheduling in LPT order: within 4/3 - 1/(3P) of the optimum
    owner, before, after, _ = orc.place_lpt(P, hist, E, everything_on_zero)
    opt = best_makespan(P, hist, E)
    assert opt <= after.max() and after.max() * 3 * P <= (4 * P - 1) * opt
    # with the limit: a valid map that is never worse than the one it replaces and never better than the optimum
    cap = -(-E // P)
    owner, before, after, migrated = orc.place_lpt(P, hist, cap, everything_on_zero)
    assert np.bincount(owner, minlength=P).max() <= cap
    assert best_makespan(P, hist, cap) <= after.max() <= before.max()
    assert after.sum() == before.sum() == hist.sum()
    assert migrated == int((owner != everything_on_zero).sum())
    # placing again changes nothing: the same bins cannot be strictly better than themselves
    again, b2, a2, m2 = orc.place_lpt(P, hist, cap, owner)
    assert np.array_equal(again, owner) and m2 == 0 and np.array_equal(b2, after) and np.array_equal(a2, after)


def test_place_lpt_keeps_what_it_cannot_improve_and_names_bins_after_ranks():
    # any map with two experts per rank pairs the 10 with a 3: 13 cannot be lowered, the map stays
    owner, before, after, migrated = orc.place_lpt(2, [10, 3, 3, 3], 2, [0, 0, 1, 1])
    assert owner.tolist() == [0, 0, 1, 1] and migrated == 0 and after.tolist() == before.tolist() == [13, 6]
    # a map that already equals the LPT bins up to the ranks' names costs no migration once it is improved on:
    # start from the bins shifted by one rank with one expert misplaced
    rng = np.random.default_rng(5)
    P, per = 4, 4
    hist = rng.choice(np.arange(1, 10000), size=P * per, replace=False).astype(np.int64)    # distinct
    base, _, base_load, _ = orc.place_lpt(P, hist, per, np.zeros(P * per, dtype=np.int32))
    shifted = (base + 1) % P
    heavy_rank = int(np.argmax(orc.rank_loads(P, shifted, hist)))
    light_rank = int(np.argmin(orc.rank_loads(P, shifted, hist)))
    worse = shifted.copy()
    a = [e for e in range(P * per) if shifted[e] == heavy_rank]
    b = [e for e in range(P * per) if shifted[e] == light_rank]
    ea, eb = min(a, key=lambda e: hist[e]), max(b, key=lambda e: hist[e])
    assert heavy_rank != light_rank and hist[eb] > hist[ea]
    worse[ea], worse[eb] = light_rank, heavy_rank                                   # heavier heavy rank
    owner, before, after, migrated = orc.place_lpt(P, hist, per, worse)
    assert before.max() > base_load.max() and sorted(after.tolist()) == sorted(base_load.tolist())
    assert np.array_equal(owner, shifted) and migrated == 2                         # the two swapped experts go back
    # relabelling the experts (distinct histories) permutes the map and leaves the loads alone
    perm = rng.permutation(P * per)
    o2, _, a2, _ = orc.place_lpt(P, hist[perm], per, np.zeros(P * per, dtype=np.int32))
    assert sorted(a2.tolist()) == sorted(base_load.tolist())
    with pytest.raises(ValueError):
        orc.place_lpt(2, [1, 2, 3], 1, [0, 0, 1])


def test_mark_dynamic_takes_each_ranks_busiest_experts():
    owner = np.array([0, 0, 0, 1, 1, 1, 2, 2], dtype=np.int32)
    hist = np.array([5, 9, 9, 1, 0, 7, 3, 3], dtype=np.int64)
    assert orc.mark_dynamic(3, owner, hist, 2).tolist() == [0, 1, 1, 1, 0, 1, 1, 1]     # ties: lowest id first
    assert orc.mark_dynamic(3, owner, hist, 1).tolist() == [0, 1, 0, 0, 0, 1, 1, 0]
    assert orc.mark_dynamic(3, owner, hist, 0).sum() == 0 and orc.mark_dynamic(3, owner, hist, 5).sum() == 8
    # on the contiguous map with history = popularity it is the workload generator's own choice
    import workloads
    wl = workloads.make("C4", T=64, d=8, f=8)
    pop = np.round(np.exp(wl.bias) * 1e6).astype(np.int64)
    assert np.array_equal(orc.mark_dynamic(wl.P, wl.owner(), pop, 4), wl.dyn_flags(4))


def test_apply_moves_gives_the_planned_loads():
    rng = np.random.default_rng(3)
    P, E = 4, 16
    owner = (np.arange(E) // 4).astype(np.int32)
    n = rng.integers(0, 500, size=E).astype(np.int64)
    flags = np.ones(E, dtype=np.uint8)
    moves, before, after = orc.plan_whole(P, owner, n, flags, np.full(P, 2), 0)
    assert moves
    home = orc.apply_moves(owner, moves)
    assert np.array_equal(orc.rank_loads(P, home, n), after)
    assert np.array_equal(orc.apply_moves(owner, []), owner)


def test_ffn_backward_is_separable_over_hidden_units_and_output_columns():
    # what the full-size GPU test relies on to reach the oracle with sampled columns: the sub-expert made of
    # some hidden units yields exactly those columns of dWg and dWu; restricting the output columns yields
    # exactly those columns of dWd
    rng = np.random.default_rng(0)
    m, d, f = 7, 12, 10
    x, dy = rng.normal(size=(m, d)), rng.normal(size=(m, d))
    wg, wu, wd = rng.normal(size=(d, f)), rng.normal(size=(d, f)), rng.normal(size=(f, d))
    _, dWg, dWu, dWd = orc.ffn_rows_backward(x, wg, wu, wd, dy)
    cols, dcols = [0, 6, 9], [1, 11]
    _, a, b, _ = orc.ffn_rows_backward(x, wg[:, cols], wu[:, cols], wd[cols, :], dy)
    c = orc.ffn_rows_backward(x, wg, wu, wd[:, dcols], dy[:, dcols])[3]
    assert np.allclose(a, dWg[:, cols], rtol=1e-13, atol=1e-13) and np.allclose(b, dWu[:, cols], rtol=1e-13, atol=1e-13)
    assert np.allclose(c, dWd[:, dcols], rtol=1e-13, atol=1e-13)
