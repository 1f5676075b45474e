"""Seeded synthetic CTR mini-batches (inputs only; none of the method's arithmetic).

The paper trains on proprietary click logs (Section 5, data description), so
every input here is synthetic and takes only the *shape* of that workload:
multi-hot sparse instances with tens to hundreds of non-zero features drawn
from a heavy-tailed popularity law (Section 2.1), a fixed number of feature
slots per instance, and a dense gradient arriving from the network above the
embedding layer (Algorithm 1, the train step between pull and push).

This module serves both the CPU oracle and the HIP path: tests generate one
batch and hand the same arrays to each side.  It imports neither of them.

Recipe per batch (all draws from one ``torch.Generator`` seeded with
``base_seed + 1000*config_id + step + 100000*replica``):

* ``offsets[G+1]``  CSR boundaries, G = B*S segments; ids per segment are
  uniform{1..8}, max(1, Poisson(3)) or Poisson(4) depending on the config.
* ranks            bounded Zipf(s) over 1..U by inverting the continuous
  power-law CDF in float64: ``floor(U**u)`` for s = 1, otherwise
  ``floor(((U**(1-s) - 1)*u + 1)**(1/(1-s)))`` with u ~ U[0,1).
* ``keys[L]``       a fixed bijection of the rank onto the config's id width
  (64, 40 or 48 bits): two rounds of odd-multiply and xor-shift modulo 2**w.
  One global key space shared by all slots.
* ``grad[G, D]``    i.i.d. N(0,1) float32, independent of the table contents.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np
import torch

_M1 = 0x9E3779B97F4A7C15
_M2 = 0xC2B2AE3D27D4EB4F


def _as_i64(v: int) -> int:
    v &= (1 << 64) - 1
    return v - (1 << 64) if v >= (1 << 63) else v


@dataclass(frozen=True)
class Workload:
    """One row of the configuration list this build is measured on."""
    config_id: int
    name: str
    capacity_rows: int          # R
    dim: int                    # D
    batch: int                  # B samples
    slots: int                  # S slots per sample
    ids_dist: str               # "uniform1_8" | "poisson3_min1" | "poisson4"
    zipf_s: float
    zipf_universe: int          # U: ranks 1..U
    key_bits: int               # w: keys live in [0, 2**w)
    n_replicas: int = 1         # W
    k_step: int = 0             # k (0 = single-table mode)
    steps: int = 1
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    init_std: float = 0.01
    load_factor: float = 0.5

    @property
    def n_segments(self) -> int:
        return self.batch * self.slots


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload(1, "tiny", 1 << 16, 8, 1024, 16, "uniform1_8", 1.1, 10 ** 6, 64, steps=1),
    "mid": Workload(2, "mid", 1 << 22, 16, 8192, 100, "poisson3_min1", 1.05, 1 << 22, 40, steps=20),
    "large": Workload(3, "large", 1 << 24, 64, 32768, 300, "poisson4", 1.0, 1 << 24, 48, steps=50),
    "kstep": Workload(4, "kstep", 1 << 22, 16, 4096, 100, "poisson3_min1", 1.05, 1 << 22, 40,
                      n_replicas=8, k_step=4, steps=40),
    # the full training step: the large table under a dense tower 19200-1024-512-256-1, batch 16384
    "full": Workload(5, "full", 1 << 24, 64, 16384, 300, "poisson4", 1.0, 1 << 24, 48, steps=50),
}
FULL_STEP_HIDDEN = (1024, 512, 256)
FULL_STEP_CLICK_RATE = 0.05


def make_labels(w: Workload, step: int, device="cpu", base_seed: int = 20220105) -> torch.Tensor:
    """Bernoulli(FULL_STEP_CLICK_RATE) click labels, float32 [B]."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(batch_seed(w, step, 7, base_seed))
    return (torch.rand(w.batch, generator=gen, device=dev) < FULL_STEP_CLICK_RATE).to(torch.float32)


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (used for reduced-size parity cases)."""
    return replace(w, **kw)


def batch_seed(w: Workload, step: int, replica: int = 0, base_seed: int = 20220105) -> int:
    return base_seed + 1000 * w.config_id + step + 100000 * replica


def _mix_rank_to_key(rank: torch.Tensor, bits: int) -> torch.Tensor:
    """Bijection of [0, 2**bits) applied to int64 ranks; result is the uint64 bit pattern."""
    x = rank.clone()
    if bits == 64:
        def lsr(t, k):
            return (t >> k) & ((1 << (64 - k)) - 1)
        x = x * _as_i64(_M1)
        x = x ^ lsr(x, 32)
        x = x * _as_i64(_M2)
        x = x ^ lsr(x, 29)
        return x
    mask = (1 << bits) - 1
    h = bits // 2
    x = (x * _as_i64(_M1)) & mask
    x = x ^ (x >> h)
    x = (x * _as_i64(_M2)) & mask
    x = x ^ (x >> (h + 1))
    return x


def zipf_ranks(n: int, s: float, universe: int, gen: torch.Generator, device) -> torch.Tensor:
    u = torch.rand(n, dtype=torch.float64, generator=gen, device=device)
    if s == 1.0:
        r = torch.pow(torch.tensor(float(universe), dtype=torch.float64, device=device), u)
    else:
        a = float(universe) ** (1.0 - s) - 1.0
        r = torch.pow(a * u + 1.0, 1.0 / (1.0 - s))
    r = torch.floor(r).to(torch.int64)
    return r.clamp_(1, universe)


def make_batch(w: Workload, step: int, replica: int = 0, device="cpu",
               base_seed: int = 20220105, with_grad: bool = True) -> Dict[str, torch.Tensor]:
    """Returns {"keys": int64[L] (uint64 bit patterns), "offsets": int32[G+1], "grad": f32[G,D]}."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(batch_seed(w, step, replica, base_seed))
    G = w.n_segments
    if w.ids_dist == "uniform1_8":
        counts = torch.randint(1, 9, (G,), generator=gen, device=dev, dtype=torch.int64)
    elif w.ids_dist == "poisson3_min1":
        lam = torch.full((G,), 3.0, dtype=torch.float32, device=dev)
        counts = torch.poisson(lam, generator=gen).to(torch.int64).clamp_(min=1)
    elif w.ids_dist == "poisson4":
        lam = torch.full((G,), 4.0, dtype=torch.float32, device=dev)
        counts = torch.poisson(lam, generator=gen).to(torch.int64)
    else:
        raise ValueError(w.ids_dist)
    offsets = torch.zeros(G + 1, dtype=torch.int64, device=dev)
    torch.cumsum(counts, 0, out=offsets[1:])
    L = int(offsets[-1].item())
    if L >= (1 << 31):
        raise ValueError("batch too large")
    ranks = zipf_ranks(L, w.zipf_s, w.zipf_universe, gen, dev)
    keys = _mix_rank_to_key(ranks, w.key_bits)
    out = {"keys": keys.contiguous(), "offsets": offsets.to(torch.int32).contiguous()}
    if with_grad:
        out["grad"] = torch.randn((G, w.dim), generator=gen, device=dev, dtype=torch.float32)
    return out


def as_numpy(batch: Dict[str, torch.Tensor]) -> Dict[str, np.ndarray]:
    """Host views with the ABI's unsigned types (keys uint64, offsets uint32)."""
    out = {
        "keys": batch["keys"].cpu().numpy().view(np.uint64),
        "offsets": batch["offsets"].cpu().numpy().view(np.uint32),
    }
    if "grad" in batch:
        out["grad"] = batch["grad"].cpu().numpy()
    return out
