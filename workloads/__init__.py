"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random inputs (update vectors, models, scheduler orders,
LDA count-delta triples).  It contains none of the method's arithmetic and is
the one piece of code shared by the tests of the CPU oracle and of the GPU
library: both sides receive the same bits from here.

The dense shapes stand in for the deep-learning updates the paper exchanges
(Sec. 2, "Performance based on model complexity": a ResNet-50 update is about
100 MB; Sec. 6 datasets) and the sparse shape for the LDA word-topic matrix
update (Sec. 6: vocabulary about 10^5 words).  No dataset is read.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np
import torch

BASE_SEED = 1907


@dataclass(frozen=True)
class DenseConfig:
    name: str
    index: int            # position in the list of configurations
    call: str             # "aggregate_apply" | "apply_ordered"
    K: int
    n: int
    dtype: str            # "f32" | "bf16"
    sigma: float
    heavy_tail: bool      # 1 % of elements scaled by 100
    lr: float
    mu: float
    momentum: bool
    weighted: bool        # weights 1/K

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def in_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def algorithmic_bytes(self, n=None) -> int:
        """Bytes the call must move: every update once, model (+ momentum)
        read and written once."""
        n = self.n if n is None else n
        state = 16 if self.momentum else 8
        return (self.in_bytes * self.K + state) * n


@dataclass(frozen=True)
class SparseConfig:
    name: str
    index: int
    V: int
    T: int
    K: int
    m: int                # triples per worker
    zipf_s: float

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    def algorithmic_bytes(self, distinct_cells: int, m=None) -> int:
        """12 bytes of triple stream per triple, one 4-byte read and one 4-byte
        write of every DISTINCT cell the batch touches (counted on the inputs by
        the caller), and the totals read and written once."""
        m = self.m if m is None else m
        return 12 * self.K * m + 8 * distinct_cells + 8 * self.T


CONFIGS = {
    "cfg1": DenseConfig("cfg1", 0, "aggregate_apply", K=4, n=1_048_576,
                        dtype="f32", sigma=0.01, heavy_tail=False, lr=0.01,
                        mu=0.0, momentum=False, weighted=True),
    "cfg2": DenseConfig("cfg2", 1, "aggregate_apply", K=16, n=25_557_032,
                        dtype="f32", sigma=0.001, heavy_tail=True, lr=0.1,
                        mu=0.9, momentum=True, weighted=True),
    "cfg3": DenseConfig("cfg3", 2, "apply_ordered", K=32, n=61_100_840,
                        dtype="f32", sigma=0.001, heavy_tail=False, lr=0.01,
                        mu=0.9, momentum=True, weighted=False),
    "cfg4": DenseConfig("cfg4", 3, "aggregate_apply", K=8, n=138_357_544,
                        dtype="bf16", sigma=0.002, heavy_tail=False, lr=0.01,
                        mu=0.9, momentum=True, weighted=True),
    "cfg5": SparseConfig("cfg5", 4, V=100_000, T=1_000, K=32, m=2_000_000,
                         zipf_s=1.1),
}


def scaled(cfg, **kw):
    """The same recipe at another size (parity tests use small n / m)."""
    return replace(cfg, **kw)


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def scheduler_order(K: int, seed: int, n_dropped: int = 0) -> np.ndarray:
    """A seeded permutation of the K workers, standing in for the order the
    scheduler hands down; the last ``n_dropped`` entries are cut off, as when
    the scheduler drops late updates."""
    perm = np.random.default_rng(seed).permutation(K).astype(np.int32)
    return perm[: K - n_dropped].copy()


def dense_update(cfg: DenseConfig, k: int, device) -> torch.Tensor:
    """Update vector of worker k: N(0, sigma^2), optionally heavy-tailed,
    optionally rounded (nearest-even) to bfloat16."""
    g = _gen(device, cfg.seed * 1000 + 17 * k + 1)
    u = torch.randn(cfg.n, generator=g, device=device, dtype=torch.float32)
    u.mul_(cfg.sigma)
    if cfg.heavy_tail:
        big = torch.rand(cfg.n, generator=g, device=device) < 0.01
        u = torch.where(big, u * 100.0, u)
    if cfg.dtype == "bf16":
        u = u.to(torch.bfloat16)
    return u.contiguous()


def dense_inputs(cfg: DenseConfig, device, momentum_init: str = "zeros",
                 n_dropped: int = 0) -> dict:
    """All inputs of one dense call.  ``momentum_init``: "zeros" (as in the
    timed run) or "random" (N(0, (lr*sigma)^2), an extra parity case)."""
    device = torch.device(device)
    updates = [dense_update(cfg, k, device) for k in range(cfg.K)]
    g = _gen(device, cfg.seed * 1000 + 999)
    model = torch.randn(cfg.n, generator=g, device=device, dtype=torch.float32)
    momentum = None
    if cfg.momentum:
        if momentum_init == "zeros":
            momentum = torch.zeros(cfg.n, device=device, dtype=torch.float32)
        else:
            momentum = torch.randn(cfg.n, generator=g, device=device,
                                   dtype=torch.float32) * (cfg.lr * cfg.sigma)
    weights = None
    if cfg.weighted:
        weights = np.full(cfg.K, 1.0 / cfg.K, dtype=np.float32)
    return {
        "updates": updates,
        "model": model,
        "momentum": momentum,
        "order": scheduler_order(cfg.K, cfg.seed, n_dropped),
        "weights": weights,
        "lr": cfg.lr,
        "mu": cfg.mu,
    }


def zipf_cdf(V: int, s: float) -> np.ndarray:
    """Cumulative distribution of the Zipf law truncated to ranks 1..V."""
    pmf = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(pmf)
    cdf /= cdf[-1]
    return cdf


def sparse_triples(cfg: SparseConfig, k: int, device, permute_ids: bool = False,
                   n_invalid: int = 0) -> torch.Tensor:
    """int32 [m, 3] buffer of (word, topic, delta) triples of worker k:
    word ~ truncated Zipf(s) by inverse CDF (word id = rank - 1, or a seeded
    permutation of the ids), topic uniform, delta = +-1 equiprobable.  The first
    ``n_invalid`` triples get an out-of-range word or topic."""
    device = torch.device(device)
    g = _gen(device, cfg.seed * 1000 + 31 * k + 7)
    cdf = torch.from_numpy(zipf_cdf(cfg.V, cfg.zipf_s)).to(device)
    u = torch.rand(cfg.m, generator=g, device=device, dtype=torch.float64)
    word = torch.searchsorted(cdf, u, right=True).clamp_(max=cfg.V - 1)
    if permute_ids:
        perm = torch.from_numpy(
            np.random.default_rng(cfg.seed + 77).permutation(cfg.V)).to(device)
        word = perm[word]
    topic = torch.randint(0, cfg.T, (cfg.m,), generator=g, device=device)
    delta = torch.randint(0, 2, (cfg.m,), generator=g, device=device) * 2 - 1
    tr = torch.stack([word, topic, delta], dim=1).to(torch.int32).contiguous()
    if n_invalid:
        bad = min(n_invalid, cfg.m)
        idx = torch.arange(bad, device=device, dtype=torch.int32)
        sel = idx % 4
        w, t = tr[:bad, 0], tr[:bad, 1]
        w = torch.where(sel == 0, cfg.V + idx, w)
        w = torch.where(sel == 1, -1 - idx, w)
        t = torch.where(sel == 2, cfg.T + idx, t)
        t = torch.where(sel == 3, -1 - idx, t)
        tr[:bad, 0], tr[:bad, 1] = w, t
    return tr


def sparse_inputs(cfg: SparseConfig, device, init: str = "zeros",
                  permute_ids: bool = False, n_invalid: int = 0) -> dict:
    """Inputs of one sparse call.  ``init``: "zeros", or "random" = seeded
    counts in [0, 50) with totals equal to their column sums."""
    device = torch.device(device)
    triples = [sparse_triples(cfg, k, device, permute_ids, n_invalid)
               for k in range(cfg.K)]
    if init == "zeros":
        counts = torch.zeros(cfg.V * cfg.T, dtype=torch.int32, device=device)
        totals = torch.zeros(cfg.T, dtype=torch.int32, device=device)
    else:
        g = _gen(device, cfg.seed * 1000 + 555)
        counts = torch.randint(0, 50, (cfg.V * cfg.T,), generator=g,
                               device=device, dtype=torch.int32)
        totals = counts.view(cfg.V, cfg.T).sum(dim=0, dtype=torch.int64).to(
            torch.int32)
    return {"counts": counts, "totals": totals, "triples": triples}


def to_host(t: torch.Tensor) -> np.ndarray:
    """Host numpy copy of a tensor; bfloat16 comes back as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()
