"""The forward FFN call that allocates nothing (feplb_grouped_ffn_static: its tile table lives in
device memory that is part of the library) against the ordinary call with a caller's workspace.
Same kernels, so every output must be bit-identical.  Needs an MI355X: run with -m gpu."""
import numpy as np
import pytest
import torch

import paper_2604_19654_amd as fe

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


def make_case(sizes, d, f, seed, k=2):
    gen = torch.Generator().manual_seed(seed)
    G = len(sizes)
    R = int(sum(sizes))
    offsets = torch.tensor(np.concatenate([[0], np.cumsum(sizes)]), dtype=torch.int32, device=DEV)
    T = max(R, 1)
    X = torch.randn((T, d), generator=gen).to(torch.bfloat16).to(DEV)
    # rows gathered through row_src: flat assignment indices t*k + j of a random token order
    order = torch.randperm(T, generator=gen)[:R]
    row_src = (order * k + torch.randint(0, k, (R,), generator=gen)).to(torch.int32).to(DEV)
    W = [tuple((torch.randn(s, generator=gen) * 0.05).to(torch.bfloat16).to(DEV) for s in ((d, f), (d, f), (f, d)))
         for _ in range(G)]
    cols = tuple([w[i] for w in W] for i in range(3))
    return R, G, offsets, X, row_src, cols


def run_both(sizes, d, f, seed, yp_dtype, pad=5):
    R, G, offsets, X, row_src, cols = make_case(sizes, d, f, seed)
    R_cap = R + pad
    outs = []
    for static in (False, True):
        H = torch.full((R_cap, f), 7.0, dtype=torch.bfloat16, device=DEV)
        Yp = torch.full((R_cap, d), 9.0, dtype=yp_dtype, device=DEV)
        if static:
            fe.feplb_grouped_ffn_static(X, offsets, 0, G, d, f, *cols, H, Yp, row_src=row_src, k=2)
        else:
            fe.feplb_grouped_ffn(X, offsets, 0, G, d, f, *cols, H, Yp, row_src=row_src, k=2)
        torch.cuda.synchronize()
        outs.append((H, Yp))
    (H0, Y0), (H1, Y1) = outs
    assert torch.equal(H0, H1) and torch.equal(Y0, Y1)
    assert (H1[R:].float() == 7.0).all() and (Y1[R:].float() == 9.0).all()     # rows past the last group untouched
    assert R == 0 or Y1[:R].float().abs().max().item() > 0
    return R


def test_static_scratch_call_equals_the_workspace_call_twice_in_a_row():
    # two calls in a row on the same GPU share the built-in table: the second is smaller, with
    # another group count and other shapes, and must not see anything of the first
    say("static-scratch FFN, first call: 9 groups, 2400 rows")
    r1 = run_both([300, 0, 513, 1, 256, 700, 0, 130, 500], 512, 256, seed=1, yp_dtype=torch.float32)
    say("static-scratch FFN, second call: 3 groups, 270 rows")
    r2 = run_both([260, 0, 10], 256, 128, seed=2, yp_dtype=torch.bfloat16)
    assert r2 < r1
    say("static-scratch FFN, third call: nothing to do")
    run_both([0, 0], 256, 128, seed=3, yp_dtype=torch.float32)


def test_static_scratch_call_phase_by_phase_and_on_a_range():
    sizes, d, f = [100, 300, 0, 257, 64], 256, 256
    R, G, offsets, X, row_src, cols = make_case(sizes, d, f, seed=4)
    H0 = torch.zeros((R, f), dtype=torch.bfloat16, device=DEV)
    Y0 = torch.zeros((R, d), dtype=torch.float32, device=DEV)
    fe.feplb_grouped_ffn(X, offsets, 0, G, d, f, *cols, H0, Y0, row_src=row_src, k=2)
    H1, Y1 = torch.zeros_like(H0), torch.zeros_like(Y0)
    # the static range and the dynamic range as two calls, the second phase by phase
    fe.feplb_grouped_ffn_static(X, offsets, 0, 2, d, f, *cols, H1, Y1, row_src=row_src, k=2)
    for ph in (fe.FFN_SCHEDULE, fe.FFN_GATE_UP, fe.FFN_DOWN):
        fe.feplb_grouped_ffn_static(X, offsets, 2, G, d, f, *cols, H1, Y1, phases=ph, row_src=row_src, k=2)
    torch.cuda.synchronize()
    assert torch.equal(H0, H1) and torch.equal(Y0, Y1)


def test_static_scratch_call_refuses_what_its_table_cannot_hold():
    L = fe.lib()
    # 5 million rows need more tile entries than 256 KiB hold: refused on the host, nothing launched
    rc = L.feplb_grouped_ffn_static(None, None, 0, 0, None, 0, 4, 5_000_000, 256, 128, None, None, None, None, None,
                                    0, 7, None)
    assert rc == -2 and b"built-in scratch" in L.feplb_last_error()
    assert fe.feplb_grouped_ffn_workspace_bytes(4_000_000, 128) <= fe.STATIC_WS_BYTES
