"""The straggler study (paper Section 3.1 Metrics, Sections 3.3 and 3.5) only sequences library
calls; its bookkeeping is checked against the oracle on the CPU, and one small run on the GPU."""
import numpy as np
import pytest

import workloads
from oracle import feplb_oracle as orc
from paper_2604_19654_amd import straggler as st


@pytest.mark.parametrize("P,dyn,seed", [(8, 4, 0), (4, 2, 1), (2, 8, 2), (8, 8, 3)])
def test_token_bookkeeping_matches_the_oracle(P, dyn, seed):
    wl = workloads.make("C4", device="cpu", seed=4000 + seed, P=P, T=P * 256, d=8, f=8)
    ids, _, counts = orc.route_topk(wl.logits.numpy(), wl.k)
    owner, flags = wl.owner(), wl.dyn_flags(dyn)
    moves, before, after = st.plan_counts(P, owner, counts, flags, dyn)
    o_moves, o_before, o_after = orc.plan_whole(P, owner, counts, flags, np.full(P, dyn, dtype=np.int32), 0)
    assert np.array_equal(before, o_before) and np.array_equal(after, o_after)
    assert st.straggler(before) == orc.token_straggler(o_before)
    assert st.straggler(after) == orc.token_straggler(o_after)
    # the whole-expert plan never raises the maximum load, so the straggler cannot grow
    assert after.max() <= before.max() and after.sum() == before.sum()
    # the shares handed to the FFN timer carry exactly the planned loads, one group per non-empty expert
    shares = st.placement(P, owner, counts, moves)
    assert [sum(s) for s in shares] == [int(x) for x in after]
    assert sum(len(s) for s in shares) == int((counts > 0).sum())
    assert [sum(s) for s in st.placement(P, owner, counts, [])] == [int(x) for x in before]


@pytest.mark.gpu
def test_small_study_runs_and_reduces_both_stragglers():
    r = st.study(P=4, dyn_list=[2, 4], n_batches=2, tokens_per_rank=4096, d=512, f=256, gemm_dyn=4)
    t = r["token_straggler"]
    assert t["before"] > 0 and t["dyn2"] <= t["before"] and t["dyn4"] <= t["dyn2"]
    g = r["gemm_straggler_ms"]
    assert g["before"] > 0 and g["dyn4"] >= 0
