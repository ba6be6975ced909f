"""The seeded input recipes: shapes, determinism, and the structure each
workload is meant to have (checked with the oracle's router)."""
import numpy as np
import torch

import workloads
from oracle import feplb_oracle as orc


def test_shapes_and_determinism():
    a = workloads.make("C1")
    b = workloads.make("C1")
    assert a.logits.shape == (512, 8) and a.X.shape == (512, 256) and a.X.dtype == torch.bfloat16
    assert torch.equal(a.logits, b.logits) and torch.equal(a.X, b.X)
    wa, wb = a.expert_weights(3), b.expert_weights(3)
    assert wa[0].shape == (256, 512) and wa[2].shape == (512, 256)
    assert all(torch.equal(x, y) for x, y in zip(wa, wb))
    assert not torch.equal(a.expert_weights(2)[0], wa[0])
    assert abs(float(wa[0].float().std()) - 0.02) < 2e-3
    assert workloads.expert_bytes(6144, 2048) == 72 * 2**20


def test_skewed_share_makes_rank0_the_straggler():
    wl = workloads.make("C3", d=8, f=8)
    _, _, counts = orc.route_topk(wl.logits.numpy(), wl.k)
    L = orc.rank_loads(wl.P, wl.owner(), counts)
    assert int(np.argmax(L)) == 0
    local = counts[wl.local_experts()]
    assert local.max() > 5 * (counts.sum() / wl.E) and (local == 0).sum() >= 4


def test_balanced_share_is_balanced_and_large_share_has_empty_experts():
    wl = workloads.make("C2", d=8, f=8)
    _, _, counts = orc.route_topk(wl.logits.numpy(), wl.k)
    local = counts[wl.local_experts()]
    assert 400 < local.min() and local.max() < 640
    wl = workloads.make("C5", d=8, f=8)
    _, _, counts = orc.route_topk(wl.logits.numpy(), wl.k)
    local = counts[wl.local_experts()]
    assert len(local) == 32 and (local == 0).sum() >= 4 and local.max() > 10000


def test_dyn_flags_pick_four_per_rank():
    wl = workloads.make("C4", T=64, d=8, f=8)
    flag = wl.dyn_flags(4)
    assert flag.reshape(8, 16).sum(axis=1).tolist() == [4] * 8


def test_popularity_seed_persists_over_micro_batches():
    a = workloads.make("C4", T=256, d=8, f=8, seed=50, pop_seed=7)
    b = workloads.make("C4", T=256, d=8, f=8, seed=51, pop_seed=7)
    c = workloads.make("C4", T=256, d=8, f=8, seed=51)
    assert np.array_equal(a.bias, b.bias) and not np.array_equal(a.logits.numpy(), b.logits.numpy())
    assert not np.array_equal(b.bias, c.bias)
    # the noise follows `seed` alone
    assert np.allclose(b.logits.numpy() - b.bias.astype(np.float32), c.logits.numpy() - c.bias.astype(np.float32), atol=1e-4)
    # without pop_seed nothing changes
    assert np.array_equal(workloads.make("C3", T=64, d=8, f=8).bias, workloads.make("C3", T=64, d=8, f=8, pop_seed=1003).bias)


def test_popularity_drifts_by_one_pair_per_swap():
    base = workloads.make("C4", T=64, d=8, f=8, seed=9, pop_seed=3)
    prev = base.bias
    for n in range(1, 6):
        cur = workloads.make("C4", T=64, d=8, f=8, seed=9 + n, pop_seed=3, drift_swaps=n).bias
        assert sorted(cur.tolist()) == sorted(base.bias.tolist())          # the same popularities, re-assigned
        assert (cur != prev).sum() in (0, 2)                                # one more pair exchanged (or a pair (i, i))
        prev = cur
