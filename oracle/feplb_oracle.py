"""CPU oracle for one EP rank's MoE hot path (FEPLB, Sections 2.2-2.3).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
GPU library is checked against.  Only the test-suite, the smoke check and the
benchmark's ``cpu_baseline`` leg may import it; the product never does, and it
imports nothing from the product.  It shares no code, table or constant with
the HIP path.

Arithmetic: float64 on the exact input values (fp32 logits, bf16 rows and
weights widened without change); nothing is rounded in between.  NumPy's
matmul and stable argsort serve as library steps; there is no tiling, fusion
or reordering.

What each function follows:
  route_topk        Section 2.3 (the router yields per-token expert choices);
                    the score is softmax over all experts, the k largest kept
                    and renormalised (the paper does not state the score).
  permute           Section 2.2 Phase 1 (tokens are permuted by expert) and
                    Section 2.3 (static / dynamic expert partition).
  ffn_rows, grouped_ffn   Section 3.1 (expert compute is a grouped GEMM);
                    the expert is a SwiGLU MLP without biases.
  ffn_rows_backward, grouped_ffn_backward   the gradients of that definition
                    (Section 3.2 reports the layer's backward time beside the
                    forward one): chain rule on y = (silu(x Wg) * (x Wu)) Wd.
  combine           Section 2.3 (combine returns expert outputs to tokens).
  combine_backward, permute_backward, route_topk_backward   the gradients of
                    combine, gather_rows and route_topk's weights (selection held
                    fixed), which with grouped_ffn_backward make up the layer's
                    backward pass of Section 3.2.
  moe_token, moe_tokens   the layer's definition per token, no permutation.
  plan_whole        Section 2.3, the greedy whole-expert balancer.
  plan_overflow     NOT in the paper (which never splits an expert's batch):
                    the replicate-the-hottest rule of the rebalanced workload.
                    Parity unpinned against the paper; invariants only.
  pick_receiver     workload convention, not in the paper.  Parity unpinned.
  token_straggler   Section 3.1 Metrics.
  history_update, place_lpt, mark_dynamic   Section 2.3, macro level: a Router
                    Predictor re-assigns experts to devices from routing history,
                    now and then.  The paper names it and gives no algorithm; the
                    rule here (exponential moving average of the counts, longest
                    processing time first under a per-device expert limit, kept
                    only when it lowers the predicted maximum, bins named so that
                    few experts migrate) is this build's reading.
  experts_per_device, dynamic_buffer_bytes   Section 2.3 worked numbers.
"""
from __future__ import annotations

import numpy as np

INT32_MAX = 2**31 - 1

PLAN_WHOLE = 0
PLAN_OVERFLOW = 1


# --------------------------------------------------------------------------
# routing
# --------------------------------------------------------------------------
def route_topk(logits: np.ndarray, k: int):
    """Per token: p = softmax(logits) over all E experts; keep the k experts
    that come first in the order (logit descending, expert id ascending);
    weight j = p[id_j] / sum of the k kept p.  Position 0 holds the largest.
    Returns ids [T,k] int32, weights [T,k] float64, counts [E] int64."""
    z = np.asarray(logits)
    T, E = z.shape
    if not (1 <= k <= E):
        raise ValueError("need 1 <= k <= E")
    if not np.all(np.isfinite(z)):
        raise ValueError("logits must be finite")
    z = z.astype(np.float64)
    # stable sort of the negated logits: descending logit, ties keep the
    # lower expert id first (-0.0 and +0.0 compare equal).
    order = np.argsort(-z, axis=1, kind="stable")
    ids = order[:, :k].astype(np.int32)
    zmax = z.max(axis=1, keepdims=True)
    ez = np.exp(z - zmax)
    p = ez / ez.sum(axis=1, keepdims=True)
    pk = np.take_along_axis(p, ids.astype(np.int64), axis=1)
    w = pk / pk.sum(axis=1, keepdims=True)
    counts = np.bincount(ids.reshape(-1), minlength=E).astype(np.int64)
    return ids, w, counts


# --------------------------------------------------------------------------
# permutation
# --------------------------------------------------------------------------
def permute(ids: np.ndarray, groups):
    """Walk the flat assignments a = t*k + j in ascending order, keeping a
    running ordinal per expert.  Assignment a goes to group g when
    groups[g] = (expert, ord_lo, ord_hi) names its expert and its ordinal lies
    in [ord_lo, ord_hi).  Rows of a group keep ascending a; groups are laid out
    in table order.  Returns offsets [G+1] int32, row_src [R] int32 (the flat
    assignment of each row), inv [T*k] int32 (row of each assignment or -1)."""
    flat = np.asarray(ids).reshape(-1)
    G = len(groups)
    by_expert = {}
    for g, (e, lo, hi) in enumerate(groups):
        by_expert.setdefault(int(e), []).append((g, int(lo), int(hi)))
    ordinal = {}
    members = [[] for _ in range(G)]
    for a in range(flat.shape[0]):
        e = int(flat[a])
        o = ordinal.get(e, 0)
        ordinal[e] = o + 1
        for (g, lo, hi) in by_expert.get(e, ()):
            if lo <= o < hi:
                members[g].append(a)
                break
    offsets = np.zeros(G + 1, dtype=np.int32)
    for g in range(G):
        offsets[g + 1] = offsets[g] + len(members[g])
    row_src = np.zeros(int(offsets[G]), dtype=np.int32)
    inv = np.full(flat.shape[0], -1, dtype=np.int32)
    r = 0
    for g in range(G):
        for a in members[g]:
            row_src[r] = a
            inv[a] = r
            r += 1
    return offsets, row_src, inv


def gather_rows(X: np.ndarray, row_src: np.ndarray, k: int) -> np.ndarray:
    """Xp[r,:] = X[row_src[r] // k, :]."""
    return X[np.asarray(row_src, dtype=np.int64) // k]


# --------------------------------------------------------------------------
# expert FFN
# --------------------------------------------------------------------------
def ffn_rows(x: np.ndarray, w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray):
    """SwiGLU expert on rows x [m,d]: a = x Wg, b = x Wu, h = a*sigmoid(a)*b,
    y = h Wd.  All float64.  Returns (h [m,f], y [m,d])."""
    x = np.asarray(x, dtype=np.float64)
    a = x @ np.asarray(w_gate, dtype=np.float64)
    b = x @ np.asarray(w_up, dtype=np.float64)
    h = a * (1.0 / (1.0 + np.exp(-a))) * b
    y = h @ np.asarray(w_down, dtype=np.float64)
    return h, y


def grouped_ffn(Xp: np.ndarray, offsets: np.ndarray, weights):
    """weights[g] = (Wg, Wu, Wd) for group g.  Rows offsets[g]..offsets[g+1]
    of Xp go through expert g.  Returns (H [R,f], Yp [R,d]) float64."""
    R = int(offsets[-1])
    d = Xp.shape[1]
    f = weights[0][0].shape[1] if len(weights) else 0
    H = np.zeros((R, f))
    Yp = np.zeros((R, d))
    for g in range(len(weights)):
        lo, hi = int(offsets[g]), int(offsets[g + 1])
        if hi > lo:
            H[lo:hi], Yp[lo:hi] = ffn_rows(Xp[lo:hi], *weights[g])
    return H, Yp


def ffn_rows_backward(x, w_gate, w_up, w_down, dy):
    """Gradients of L = sum(y * dy) for y = ffn_rows(x, Wg, Wu, Wd)[1], by the
    chain rule in float64.  With a = x Wg, b = x Wu, s = sigmoid(a):
      dh = dy Wd^T;   db = dh * a * s;   da = dh * b * s * (1 + a (1 - s));
      dx = da Wg^T + db Wu^T;   dWg = x^T da;   dWu = x^T db;   dWd = h^T dy.
    Returns (dx [m,d], dWg [d,f], dWu [d,f], dWd [f,d])."""
    x = np.asarray(x, dtype=np.float64)
    wg = np.asarray(w_gate, dtype=np.float64)
    wu = np.asarray(w_up, dtype=np.float64)
    wd = np.asarray(w_down, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    a = x @ wg
    b = x @ wu
    s = 1.0 / (1.0 + np.exp(-a))
    h = a * s * b
    dh = dy @ wd.T
    db = dh * a * s
    da = dh * b * s * (1.0 + a * (1.0 - s))
    dx = da @ wg.T + db @ wu.T
    return dx, x.T @ da, x.T @ db, h.T @ dy


def grouped_ffn_backward(Xp, offsets, weights, dYp):
    """Per group g, ffn_rows_backward on rows offsets[g]..offsets[g+1] with the
    group's own matrices.  A group without rows has zero weight gradients.
    Returns (dXp [R,d], [(dWg, dWu, dWd) per group])."""
    R = int(offsets[-1])
    d = Xp.shape[1]
    dXp = np.zeros((R, d))
    grads = []
    for g in range(len(weights)):
        lo, hi = int(offsets[g]), int(offsets[g + 1])
        wg, wu, wd = weights[g]
        if hi > lo:
            dx, dwg, dwu, dwd = ffn_rows_backward(Xp[lo:hi], wg, wu, wd, dYp[lo:hi])
            dXp[lo:hi] = dx
            grads.append((dwg, dwu, dwd))
        else:
            grads.append((np.zeros(wg.shape), np.zeros(wu.shape), np.zeros(wd.shape)))
    return dXp, grads


# --------------------------------------------------------------------------
# combine
# --------------------------------------------------------------------------
def combine(Yp: np.ndarray, inv: np.ndarray, w: np.ndarray, T: int, k: int) -> np.ndarray:
    """Y[t,:] = sum over slots j with inv[t,j] >= 0 of w[t,j] * Yp[inv[t,j],:];
    a token with no local slot gets zeros."""
    d = Yp.shape[1]
    inv2 = np.asarray(inv).reshape(T, k)
    w2 = np.asarray(w, dtype=np.float64).reshape(T, k)
    Y = np.zeros((T, d))
    for j in range(k):
        sel = np.nonzero(inv2[:, j] >= 0)[0]
        Y[sel] += w2[sel, j][:, None] * Yp[inv2[sel, j]]
    return Y


def combine_backward(dY: np.ndarray, Yp: np.ndarray, inv: np.ndarray, w: np.ndarray, T: int, k: int):
    """Gradients of L = sum(Y * dY), Y = combine(Yp, inv, w): every permuted row r
    is slot (t, j) of exactly one token, so dYp[r,:] = w[t,j] * dY[t,:]; and
    dw[t,j] = <dY[t,:], Yp[inv[t,j],:]> for a local slot, 0 for the others.
    Returns (dYp [R,d], dw [T,k])."""
    dY = np.asarray(dY, dtype=np.float64)
    Yp = np.asarray(Yp, dtype=np.float64)
    inv2 = np.asarray(inv).reshape(T, k)
    w2 = np.asarray(w, dtype=np.float64).reshape(T, k)
    dYp = np.zeros_like(Yp)
    dw = np.zeros((T, k))
    for j in range(k):
        sel = np.nonzero(inv2[:, j] >= 0)[0]
        rows = inv2[sel, j]
        dYp[rows] = w2[sel, j][:, None] * dY[sel]
        dw[sel, j] = np.einsum("ij,ij->i", dY[sel], Yp[rows])
    return dYp, dw


def permute_backward(dXp: np.ndarray, inv: np.ndarray, T: int, k: int) -> np.ndarray:
    """Gradient of the row gather Xp[r,:] = X[row_src[r] // k, :]: token t receives the
    sum of the gradients of the rows that are its copies, dX[t,:] = sum over local slots j
    of dXp[inv[t,j],:]."""
    return combine(np.asarray(dXp, dtype=np.float64), inv, np.ones((T, k)), T, k)


def route_topk_backward(logits: np.ndarray, ids: np.ndarray, dw: np.ndarray) -> np.ndarray:
    """Gradient of the k routing weights with respect to the logits, the selection held
    fixed: the weights are the softmax of the k kept logits, so for a kept expert
    dz[ids_j] = w_j (dw_j - sum_i w_i dw_i), and 0 for every other expert.
    Returns dlogits [T,E] float64."""
    z = np.asarray(logits, dtype=np.float64)
    ids = np.asarray(ids)
    dw = np.asarray(dw, dtype=np.float64)
    T, E = z.shape
    kept = np.take_along_axis(z, ids.astype(np.int64), axis=1)
    ex = np.exp(kept - kept.max(axis=1, keepdims=True))
    wk = ex / ex.sum(axis=1, keepdims=True)
    inner = (wk * dw).sum(axis=1, keepdims=True)
    out = np.zeros((T, E))
    np.put_along_axis(out, ids.astype(np.int64), wk * (dw - inner), axis=1)
    return out


def moe_token(x_t: np.ndarray, ids_t, w_t, expert_weights: dict) -> np.ndarray:
    """The layer's definition for one token, with no permutation at all:
    sum over the token's k slots whose expert is in `expert_weights`
    (expert id -> (Wg, Wu, Wd)) of w_j * FFN_{e_j}(x_t)."""
    x = np.asarray(x_t, dtype=np.float64)[None, :]
    y = np.zeros(x.shape[1])
    for j in range(len(ids_t)):
        e = int(ids_t[j])
        if e in expert_weights:
            y += float(w_t[j]) * ffn_rows(x, *expert_weights[e])[1][0]
    return y


def moe_tokens(x_rows: np.ndarray, ids_rows, w_rows, keep_rows, weights_of) -> np.ndarray:
    """moe_token for a batch of tokens, visiting one expert at a time so that
    each expert's matrices are widened to float64 once.  keep_rows [m,k] marks
    the slots that are local (inv >= 0); for every expert e that occurs in a
    kept slot, the rows whose kept slot j names e get w_j * FFN_e(x) added.
    `weights_of(e)` returns (Wg, Wu, Wd).  Same sums as moe_token."""
    x = np.asarray(x_rows, dtype=np.float64)
    ids_rows = np.asarray(ids_rows)
    keep_rows = np.asarray(keep_rows, dtype=bool)
    w_rows = np.asarray(w_rows, dtype=np.float64)
    out = np.zeros_like(x)
    for e in sorted(set(int(v) for v in ids_rows[keep_rows])):
        tok, slot = np.nonzero((ids_rows == e) & keep_rows)
        y = ffn_rows(x[tok], *weights_of(e))[1]
        for i in range(tok.size):
            out[tok[i]] += w_rows[tok[i], slot[i]] * y[i]
    return out


# --------------------------------------------------------------------------
# host-side rebalancing plan
# --------------------------------------------------------------------------
def rank_loads(P: int, owner, n) -> np.ndarray:
    L = np.zeros(P, dtype=np.int64)
    for e in range(len(n)):
        L[int(owner[e])] += int(n[e])
    return L


def plan_whole(P, owner, n, dyn_flag, slots, tau):
    """Greedy whole-expert balancer.  Repeat: take the most loaded rank (lowest
    id on ties); its dynamic, not yet moved experts with at least max(tau, 1)
    rows, busiest first (lowest id on ties); the least loaded other rank that
    still has a free slot (lowest id on ties).  Move the first such expert whose
    whole batch leaves the receiver strictly below the sender's current load;
    stop when there is none.  A moved expert stays where it lands.
    Returns (moves, load_before, load_after); a move is
    (expert, src, dst, rows, ord_lo=0)."""
    E = len(n)
    L = rank_loads(P, owner, n)
    before = L.copy()
    free = [int(s) for s in slots]
    moved = [False] * E
    moves = []
    thr = max(int(tau), 1)
    while True:
        src = 0
        for r in range(1, P):
            if L[r] > L[src]:
                src = r
        dst = -1
        for r in range(P):
            if r != src and free[r] > 0 and (dst < 0 or L[r] < L[dst]):
                dst = r
        if dst < 0:
            break
        cand = [e for e in range(E)
                if int(owner[e]) == src and dyn_flag[e] and not moved[e] and int(n[e]) >= thr]
        cand.sort(key=lambda e: (-int(n[e]), e))
        pick = -1
        for e in cand:
            if L[dst] + int(n[e]) < L[src]:
                pick = e
                break
        if pick < 0:
            break
        L[src] -= int(n[pick])
        L[dst] += int(n[pick])
        free[dst] -= 1
        moved[pick] = True
        moves.append((pick, src, dst, int(n[pick]), 0))
    return moves, before, L


def pick_receiver(P, owner, n) -> int:
    """Rank whose own load is closest to half the balanced mean M = ceil(sum n / P),
    i.e. argmin |2 L[r] - M| (lowest id on ties): about half of what it will
    run is its own static work, the other half arrives as replicas."""
    L = rank_loads(P, owner, n)
    M = -(-int(np.sum(n)) // P)
    best = 0
    for r in range(1, P):
        if abs(2 * int(L[r]) - M) < abs(2 * int(L[best]) - M):
            best = r
    return best


def plan_overflow(P, owner, n, dyn_flag, slots, this_rank):
    """Replicate the hottest foreign dynamic experts on `this_rank` and give it
    the tail of their rows, up to the balanced mean M = ceil(sum n / P).
    hot = the slots[this_rank] dynamic experts not owned here with the most rows
    (lowest id on ties); spare S = max(0, M - L[this_rank]); replica i takes
    rows_i = min(n_i, floor(S * n_i / sum over hot of n)) rows, namely the LAST
    rows_i occurrences of that expert in flat order (ord_lo = n_i - rows_i)."""
    E = len(n)
    L = rank_loads(P, owner, n)
    before = L.copy()
    M = -(-int(np.sum(n)) // P)
    S = max(0, M - int(L[this_rank]))
    cand = [e for e in range(E) if dyn_flag[e] and int(owner[e]) != this_rank]
    cand.sort(key=lambda e: (-int(n[e]), e))
    hot = cand[: int(slots[this_rank])]
    tot = sum(int(n[e]) for e in hot)
    moves = []
    for e in hot:
        rows = min(int(n[e]), (S * int(n[e])) // tot) if tot > 0 else 0
        moves.append((e, int(owner[e]), this_rank, rows, int(n[e]) - rows))
        L[int(owner[e])] -= rows
        L[this_rank] += rows
    return moves, before, L


def token_straggler(loads) -> float:
    """max over ranks of the token count minus the mean (Section 3.1 Metrics)."""
    L = np.asarray(loads, dtype=np.float64)
    return float(L.max() - L.mean())


# --------------------------------------------------------------------------
# macro level: placement from routing history
# --------------------------------------------------------------------------
HIST_FRAC_BITS = 16


def history_update(hist, n, shift: int) -> np.ndarray:
    """Exponential moving average of the per-expert counts in fixed point (units of
    2^-16 rows, so that every device computes the same integers):
        hist[e] <- hist[e] + floor(((n[e] << 16) - hist[e]) / 2^shift),
    i.e. decay 1 - 2^-shift per micro-batch; shift = 0 keeps the last batch only."""
    if shift < 0 or shift > 30:
        raise ValueError("shift out of range")
    out = np.zeros(len(n), dtype=np.int64)
    for e in range(len(n)):
        h = int(hist[e])
        out[e] = h + (((int(n[e]) << HIST_FRAC_BITS) - h) // (1 << shift))     # Python's // floors
    return out


def place_lpt(P: int, hist, cap: int, owner_in):
    """New expert -> rank map from the history.  Longest processing time first: experts in
    order of history, largest first (lowest id on ties), each to the bin with the least
    accumulated history among the bins that hold fewer than `cap` experts (lowest bin on
    ties).  The result replaces the current map only if its largest bin is strictly below the
    current map's largest rank load (migration costs a weight transfer per expert).  Bins
    are then named after ranks so that many experts stay: repeatedly give the (bin, rank)
    pair that shares the most experts, among bins and ranks not yet paired (lowest bin, then
    lowest rank on ties), to each other.
    Returns (owner_out [E] int32, load_before [P], load_after [P], migrated)."""
    E = len(hist)
    if cap * P < E:
        raise ValueError("cap * P < E")
    owner_in = np.asarray(owner_in, dtype=np.int32)
    before = rank_loads(P, owner_in, hist)
    order = sorted(range(E), key=lambda e: (-int(hist[e]), e))
    load = [0] * P
    held = [0] * P
    bin_of = [0] * E
    for e in order:
        best = -1
        for b in range(P):
            if held[b] < cap and (best < 0 or load[b] < load[best]):
                best = b
        bin_of[e] = best
        load[best] += int(hist[e])
        held[best] += 1
    if E == 0 or max(load) >= int(before.max()):
        return owner_in.copy(), before, before.copy(), 0
    shared = [[0] * P for _ in range(P)]
    for e in range(E):
        shared[bin_of[e]][int(owner_in[e])] += 1
    rank_of = [-1] * P
    taken = [False] * P
    for _ in range(P):
        pick = None
        for b in range(P):
            if rank_of[b] >= 0:
                continue
            for r in range(P):
                if not taken[r] and (pick is None or shared[b][r] > shared[pick[0]][pick[1]]):
                    pick = (b, r)
        rank_of[pick[0]] = pick[1]
        taken[pick[1]] = True
    owner_out = np.array([rank_of[bin_of[e]] for e in range(E)], dtype=np.int32)
    after = rank_loads(P, owner_out, hist)
    return owner_out, before, after, int((owner_out != owner_in).sum())


def mark_dynamic(P: int, owner, hist, dyn: int) -> np.ndarray:
    """[E] uint8: on every rank its `dyn` experts with the largest history (lowest id on
    ties) are the dynamic ones (Section 2.3 gives only their number)."""
    E = len(hist)
    flag = np.zeros(E, dtype=np.uint8)
    for r in range(P):
        mine = [e for e in range(E) if int(owner[e]) == r]
        mine.sort(key=lambda e: (-int(hist[e]), e))
        for e in mine[:dyn]:
            flag[e] = 1
    return flag


def apply_moves(owner, moves) -> np.ndarray:
    """Rank that runs each expert once the whole-expert moves of a plan are applied."""
    home = np.asarray(owner, dtype=np.int32).copy()
    for (e, _src, dst, _rows, _lo) in moves:
        home[int(e)] = int(dst)
    return home


def experts_per_device(E: int, ep: int) -> int:
    return E // ep


def static_dynamic_split(E: int, ep: int, dyn: int):
    """(static, dynamic) experts per device for a given dyn (Section 2.3)."""
    per = experts_per_device(E, ep)
    return per - dyn, dyn


def dynamic_buffer_bytes(max_num_dyn: int, d: int, f: int, elem_bytes: int = 2) -> int:
    """max_num_dyn x W_expert, an expert being gate [d,f], up [d,f], down [f,d]."""
    return max_num_dyn * 3 * d * f * elem_bytes
