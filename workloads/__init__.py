"""Seeded synthetic inputs for one EP rank's share of an MoE layer.

This module only draws random numbers and shapes them into the tensors the
MoE hot path consumes (router logits, token rows, expert weights).  It holds
none of the method's arithmetic: no routing, no permutation, no FFN, no plan.
Both the CPU oracle's tests and the HIP path's tests/benchmark import it, and
it imports neither of them.

The five named workloads stand in for the routing traces of the paper's
evaluation (Section 3.1: 128 routed experts, top-k routing without auxiliary
loss, EP = 8 / 4 so 16 / 32 experts per device), which are not public.  Large
arrays are drawn with a seeded ``torch.Generator`` on the requested device (the
GPU for full-size runs; the same bits are then copied to the host for the
oracle).  The small arrays that decide the popularity of the experts are drawn
with NumPy on the host so that they do not depend on the device.

Draw order per workload, seed ``s = 1000 + c`` for workload ``Cc``:
popularity (permutation or Dirichlet, NumPy, seed s) -> logit noise (torch,
seed s) -> token rows X (torch, seed s + 1) -> expert e's weights (torch,
seed ``(s + 2) * 4096 + e``, gate then up then down), drawn on demand so that
only the experts a rank actually runs are ever materialised.  With ``pop_seed=``
the popularity is drawn from that seed instead, so that a series of micro-batches
(seeds s, s+1, ...) shares one popularity, as the batches of one training run do;
``drift_swaps=n`` exchanges the popularity ranks of n random expert pairs on top,
so that batch b with ``drift_swaps=b*m`` sees a popularity that moves by m pairs per batch.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np
import torch

__all__ = ["Workload", "make", "NAMES", "expert_bytes"]

NAMES = ("C1", "C2", "C3", "C4", "C5")

# name: (T, d, f, E, k, P ranks, local rank, popularity, n_dyn)
_SHAPES = {
    "C1": dict(T=512, d=256, f=512, E=8, k=2, P=1, rank=0, pop="uniform", n_dyn=0),
    "C2": dict(T=8192, d=4096, f=1536, E=128, k=8, P=8, rank=0, pop="uniform", n_dyn=0),
    "C3": dict(T=8192, d=4096, f=1536, E=128, k=8, P=8, rank=0, pop="zipf", n_dyn=0),
    # eight simulated ranks of 16384 tokens each: after dispatch the receiving
    # rank sees assignments from all of them, so T = 8 * 16384.
    "C4": dict(T=8 * 16384, d=6144, f=2048, E=128, k=8, P=8, rank=-1, pop="zipf", n_dyn=4),
    "C5": dict(T=32768, d=7168, f=2048, E=128, k=8, P=4, rank=0, pop="dirichlet", n_dyn=0),
}


def expert_bytes(d: int, f: int) -> int:
    """Bytes of one expert's three bf16 matrices (gate [d,f], up [d,f], down [f,d])."""
    return 3 * d * f * 2


@dataclass
class Workload:
    name: str
    seed: int
    T: int
    d: int
    f: int
    E: int
    k: int
    P: int                      # EP ranks simulated on the host
    rank: int                   # this rank, or -1 when the plan picks the receiver
    n_dyn: int                  # dynamic (replicated) expert slots on this rank
    pop: str
    device: torch.device
    bias: np.ndarray            # [E] float64, added to the logit noise
    swapped_block: int          # column block exchanged with block 0 (-1: none)
    logits: torch.Tensor        # [T,E] fp32
    X: torch.Tensor             # [T,d] bf16
    w_std: float = 0.02
    _wcache: Dict[int, Tuple[torch.Tensor, torch.Tensor, torch.Tensor]] = field(default_factory=dict)

    @property
    def experts_per_rank(self) -> int:
        return self.E // self.P

    def owner(self) -> np.ndarray:
        """Static expert -> rank map: contiguous blocks of E/P experts (Section 2.3)."""
        return (np.arange(self.E) // self.experts_per_rank).astype(np.int32)

    def local_experts(self, rank: Optional[int] = None) -> np.ndarray:
        r = self.rank if rank is None else rank
        if r < 0:
            raise ValueError("this workload's rank is chosen by the plan; pass rank=")
        n = self.experts_per_rank
        return np.arange(r * n, (r + 1) * n, dtype=np.int32)

    def dyn_flags(self, dyn: int = 4) -> np.ndarray:
        """[E] uint8: on every rank the `dyn` experts with the largest logit bias
        (lowest id on ties) are the dynamic ones (Section 2.3 gives only their
        number; imbalance comes from a few busy experts, Section 3.5)."""
        flag = np.zeros(self.E, dtype=np.uint8)
        per = self.experts_per_rank
        for r in range(self.P):
            ex = np.arange(r * per, (r + 1) * per)
            flag[ex[np.argsort(-self.bias[ex], kind="stable")[:dyn]]] = 1
        return flag

    def expert_weights(self, e: int):
        """(W_gate [d,f], W_up [d,f], W_down [f,d]) bf16 ~ N(0, 0.02), row-major."""
        e = int(e)
        if e not in self._wcache:
            g = torch.Generator(device=self.device)
            g.manual_seed((self.seed + 2) * 4096 + e)
            mats = []
            for shape in ((self.d, self.f), (self.d, self.f), (self.f, self.d)):
                w = torch.empty(shape, dtype=torch.float32, device=self.device)
                w.normal_(0.0, self.w_std, generator=g)
                mats.append(w.to(torch.bfloat16))
            self._wcache[e] = tuple(mats)
        return self._wcache[e]

    def drop_weights(self):
        self._wcache.clear()


def _zipf_bias(E: int, rng: np.random.Generator, drift_swaps: int = 0):
    """b_e = 2.0 * ln(rank_e ** -1.2), rank_e a seeded permutation of 1..E.  With drift_swaps > 0 that
    many random pairs of experts then exchange their popularity ranks, one pair after the other, drawn
    from the same generator: the popularity after n swaps is the one after n - 1 with one more pair
    exchanged, so a series of growing counts is a popularity that drifts."""
    rank_e = rng.permutation(E) + 1
    for _ in range(drift_swaps):
        i, j = rng.integers(0, E, size=2)
        rank_e[i], rank_e[j] = rank_e[j], rank_e[i]
    return 2.0 * np.log(rank_e.astype(np.float64) ** -1.2), rank_e


def _inclusion(p: np.ndarray, k: int) -> np.ndarray:
    """Inclusion probabilities of drawing k of E items without replacement with
    probability proportional to size (the survey-sampling formula
    pi_e = min(1, lam * p_e) with sum pi = k).  An expert cannot receive more
    than one pick per token, so the few most popular experts saturate at one
    and a block's expected load is T * sum of pi over its experts.  Used only to
    decide which column block is relabelled as rank 0."""
    p = np.asarray(p, dtype=np.float64)
    p = p / p.sum()
    capped = np.zeros(p.shape[0], dtype=bool)
    while True:
        lam = (k - capped.sum()) / p[~capped].sum()
        new = (~capped) & (lam * p >= 1.0)
        if not new.any():
            break
        capped |= new
    return np.where(capped, 1.0, lam * p)


def make(name: str, device="cpu", **override) -> Workload:
    """Build workload ``name`` (C1..C5); keyword overrides (T=, d=, f=, seed=, ...)
    give reduced-size variants with the same structure for the parity tests."""
    if name not in _SHAPES:
        raise KeyError(name)
    p = dict(_SHAPES[name])
    seed = int(override.pop("seed", 1000 + int(name[1:])))
    # the experts' popularity may keep its own seed while the logit noise, tokens and weights
    # follow `seed`: micro-batches of one training run share a popularity and differ in the rest
    pop_seed = int(override.pop("pop_seed", seed))
    drift_swaps = int(override.pop("drift_swaps", 0))     # Zipf popularity only: see _zipf_bias
    p.update(override)
    T, d, f, E, k, P = (int(p[x]) for x in ("T", "d", "f", "E", "k", "P"))
    if E % P:
        raise ValueError("E must be a multiple of P")
    dev = torch.device(device)
    rng = np.random.default_rng(pop_seed)
    per = E // P

    swapped = -1
    if p["pop"] == "uniform":
        bias = np.zeros(E)
    elif p["pop"] == "zipf":
        bias, rank_e = _zipf_bias(E, rng, drift_swaps)
        if p["rank"] == 0:
            # Make rank 0 the rank with the most popular experts by relabelling,
            # not by re-drawing: exchange column block 0 with the block whose
            # expected share of the k picks is largest (lowest block on ties).
            # A pure function of the drawn permutation; see _inclusion().
            mass = _inclusion(np.exp(bias), k).reshape(P, per).sum(axis=1)
            hot = int(np.argmax(mass))
            if hot != 0:
                b = bias.reshape(P, per).copy()
                b[[0, hot]] = b[[hot, 0]]
                bias = b.reshape(E)
                swapped = hot
    elif p["pop"] == "dirichlet":
        pe = rng.dirichlet(np.full(E, 0.3))
        bias = np.log(np.maximum(pe, 1e-30))
    else:
        raise ValueError(p["pop"])

    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    logits = torch.empty((T, E), dtype=torch.float32, device=dev)
    logits.normal_(0.0, 1.0, generator=g)
    logits += torch.from_numpy(bias.astype(np.float32)).to(dev)

    g.manual_seed(seed + 1)
    X = torch.empty((T, d), dtype=torch.float32, device=dev)
    X.normal_(0.0, 1.0, generator=g)
    X = X.to(torch.bfloat16)

    return Workload(name=name, seed=seed, T=T, d=d, f=f, E=E, k=k, P=P,
                    rank=int(p["rank"]), n_dyn=int(p["n_dyn"]), pop=p["pop"],
                    device=dev, bias=bias, swapped_block=swapped,
                    logits=logits, X=X)
