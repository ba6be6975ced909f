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


def oracle_counts(P, T, seed, pop_seed=None, drift_swaps=0):
    """The same micro-batch as the study's, routed by the oracle on the host (the generator's
    bits do not depend on the device for the host-drawn popularity; the logit noise is drawn
    on the device the study uses, so the caller passes that device's logits where it matters)."""
    kw = {} if pop_seed is None else {"pop_seed": pop_seed, "drift_swaps": drift_swaps}
    return workloads.make("C4", device="cuda:0", seed=seed, P=P, T=T, d=8, f=8, **kw)


@pytest.mark.gpu
def test_small_study_runs_and_reduces_both_stragglers():
    P, tokens = 4, 4096
    r = st.study(P=P, dyn_list=[2, 4], n_batches=2, tokens_per_rank=tokens, d=512, f=256, gemm_dyn=4, keep_records=True)
    t = r["token_straggler"]
    assert t["before"] > 0 and t["dyn2"] <= t["before"] and t["dyn4"] <= t["dyn2"]
    g = r["gemm_straggler_ms"]
    assert g["before"] > 0 and g["dyn4"] >= 0
    # the oracle's leg: the same logits routed, planned and measured on the CPU
    means = {"before": [], "dyn2": [], "dyn4": []}
    for rec in r["records"]:
        wl = oracle_counts(P, P * tokens, rec["seed"])
        _, _, counts = orc.route_topk(wl.logits.cpu().numpy(), wl.k)
        assert np.array_equal(rec["counts"], counts)
        for dyn in (2, 4):
            _, before, after = orc.plan_whole(P, wl.owner(), counts, wl.dyn_flags(dyn), np.full(P, dyn, dtype=np.int32), 0)
            assert np.array_equal(rec["loads"]["before"], before) and np.array_equal(rec["loads"][f"dyn{dyn}"], after)
            assert rec["token_straggler"][f"dyn{dyn}"] == orc.token_straggler(after)
        assert rec["token_straggler"]["before"] == orc.token_straggler(before)
        means["before"].append(orc.token_straggler(before))
        for dyn in (2, 4):
            means[f"dyn{dyn}"].append(rec["token_straggler"][f"dyn{dyn}"])
    for key, v in means.items():
        assert t[key] == float(np.mean(v))


@pytest.mark.gpu
def test_predictor_study_matches_the_oracle_and_the_placement_helps():
    P, tokens, dyn, warm, shift, seed0, drift = 4, 4096, 4, 3, 2, 7100, 1
    r = st.predictor_study(P=P, dyn=dyn, n_batches=warm + 3, warm=warm, shift=shift, tokens_per_rank=tokens,
                           d=512, f=256, seed0=seed0, keep_records=True, drift=drift, replace_every=2)
    # oracle leg: route every batch on the CPU, keep the history, place, plan
    E = 128
    hist = np.zeros(E, dtype=np.int64)
    slots = np.full(P, dyn, dtype=np.int32)
    owner1 = None
    recs = iter(r["records"])
    for b in range(warm + 3):
        wl = oracle_counts(P, P * tokens, seed0 + b, pop_seed=seed0, drift_swaps=b * drift)
        _, _, counts = orc.route_topk(wl.logits.cpu().numpy(), wl.k)
        if b < warm:
            hist = orc.history_update(hist, counts, shift if b else 0)
            continue
        if owner1 is None:
            owner1, pb, pa, migrated = orc.place_lpt(P, hist, E // P, wl.owner())
            assert r["placed"]["placements"][0] == (b, migrated)
            assert np.array_equal(r["placed"]["hist"], hist)
            total_migrated = migrated
            assert np.bincount(owner1, minlength=P).tolist() == [E // P] * P
        rec = next(recs)
        assert np.array_equal(rec["counts"], counts)
        for name, owner in (("contiguous", wl.owner()), ("placed", owner1)):
            flags = orc.mark_dynamic(P, owner, hist, dyn)
            _, before, after = orc.plan_whole(P, owner, counts, flags, slots, 0)
            assert np.array_equal(rec["loads"][name], before) and np.array_equal(rec["loads"][name + "+plan"], after)
            assert rec["token_straggler"][name] == orc.token_straggler(before)
            assert rec["token_straggler"][name + "+plan"] == orc.token_straggler(after)
        hist = orc.history_update(hist, counts, shift)
        if (b - warm + 1) % 2 == 0 and b + 1 < warm + 3:                       # replace_every = 2
            owner1, _, _, migrated = orc.place_lpt(P, hist, E // P, owner1)
            total_migrated += migrated
    assert np.array_equal(r["placed"]["owner"], owner1) and r["migrated_experts"] == total_migrated
    t = r["token_straggler"]
    # a popularity that persists is what the placement learns: it must beat the contiguous map on the later batches
    assert t["placed"] < t["contiguous"] and t["placed+plan"] <= t["placed"] and t["contiguous+plan"] <= t["contiguous"]
    assert r["predicted_max_load_rows"]["placed"] < r["predicted_max_load_rows"]["contiguous"]
    assert all(v >= 0 for v in r["gemm_straggler_ms"].values())
