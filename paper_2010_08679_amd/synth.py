"""Seeded synthetic inputs: embedding tables and sparse lookup index streams.

This module only draws inputs.  It holds none of the checkpoint method's arithmetic (no bitmap,
no quantizer) and is the one piece of code that both the GPU path's callers and the CPU oracle's
callers use, so that both sides see the same arrays.  Everything is a ``torch`` tensor on the
device asked for; a given (seed, device type) always gives the same values.

The shapes stand in for production recommendation models (Section 2.1: tables of many millions
of fp32 vectors of dimension such as 64; Section 3.3: about a quarter of the vectors modified per
checkpoint interval), which are not public.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    """Shape of one benchmark configuration (one entry per table is implied by ``n_tables``)."""
    name: str
    n_tables: int
    n_rows: int
    dim: int
    values: str            # "normal" | "outlier_mix"
    sigma: float
    bits: tuple
    range_mode: str        # "minmax" | "greedy"
    lookups: str           # how the dirty set is produced
    zipf_s: float = 0.0
    batch: int = 0
    pooling: int = 0
    iterations: int = 0
    dirty_fraction: float = 0.0
    num_bins: int = 0
    ratio: float = 1.0


WORKLOADS = {
    "cfg1": Workload("cfg1", 1, 100_000, 64, "normal", 0.01, (4,), "minmax", "zipf_batches",
                     zipf_s=1.05, batch=4096, pooling=1, iterations=1),
    "cfg2": Workload("cfg2", 8, 1_000_000, 128, "normal", 0.05, (4,), "minmax", "zipf_batches",
                     zipf_s=1.1, batch=2048, pooling=20, iterations=200),
    "cfg3": Workload("cfg3", 1, 40_000_000, 128, "normal", 0.05, (2, 3), "minmax",
                     "zipf_until_coverage", zipf_s=1.2, dirty_fraction=0.10),
    "cfg4": Workload("cfg4", 8, 5_000_000, 64, "outlier_mix", 0.02, (4,), "greedy",
                     "bernoulli", dirty_fraction=0.30, num_bins=100, ratio=1.0),
    "cfg5": Workload("cfg5", 12, 32_000_000, 128, "normal", 0.05, (8, 4), "minmax",
                     "zipf_batches", zipf_s=1.05, batch=4096, pooling=32, iterations=1000,
                     dirty_fraction=0.25),
}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


# ------------------------------------------------------------------------------- tables

def table_normal(n_rows: int, dim: int, sigma: float, seed: int, device="cpu") -> torch.Tensor:
    """fp32 [n_rows, dim], elements N(0, sigma) (sigma is the standard deviation)."""
    g = _gen(seed, device)
    t = torch.empty((n_rows, dim), dtype=torch.float32, device=device)
    t.normal_(0.0, sigma, generator=g)
    return t


def table_outlier_mix(n_rows: int, dim: int, sigma: float, seed: int, device="cpu",
                      outlier_p: float = 0.01, laplace_b: float = 0.2,
                      chunk_rows: int = 1 << 20) -> torch.Tensor:
    """fp32 [n_rows, dim]: each element N(0, sigma) with probability 1 - outlier_p, else
    Laplace(0, laplace_b).  Drawn chunk by chunk to bound temporary memory."""
    g = _gen(seed, device)
    t = torch.empty((n_rows, dim), dtype=torch.float32, device=device)
    for r0 in range(0, n_rows, chunk_rows):
        r1 = min(n_rows, r0 + chunk_rows)
        v = t[r0:r1]
        v.normal_(0.0, sigma, generator=g)
        pick = torch.rand(v.shape, device=device, generator=g) < outlier_p
        u = torch.rand(v.shape, device=device, generator=g) - 0.5
        lap = -laplace_b * torch.sign(u) * torch.log1p(-2.0 * u.abs().clamp(max=0.4999999))
        v.copy_(torch.where(pick, lap, v))
    return t


def make_table(w: Workload, table_index: int, seed: int, device="cpu",
               n_rows: int | None = None) -> torch.Tensor:
    rows = w.n_rows if n_rows is None else n_rows
    s = seed * 1000 + 17 * table_index + 1
    if w.values == "normal":
        return table_normal(rows, w.dim, w.sigma, s, device)
    if w.values == "outlier_mix":
        return table_outlier_mix(rows, w.dim, w.sigma, s, device)
    raise ValueError(w.values)


# ------------------------------------------------------------------------------- lookups

class ZipfSampler:
    """Bounded Zipf(s) over ranks 1..n_rows (P(k) proportional to k**-s) by inverse CDF, with a
    per-table pseudorandom rank -> row bijection so that hot rows are spread over the table."""

    def __init__(self, n_rows: int, s: float, seed: int, device="cpu",
                 explicit_perm_limit: int = 8_000_000):
        self.n_rows = int(n_rows)
        self.device = device
        k = torch.arange(1, n_rows + 1, dtype=torch.float64, device=device)
        cdf = torch.cumsum(k.pow_(-float(s)), dim=0)
        self.cdf = cdf / cdf[-1]
        del k
        self.g = _gen(seed, device)
        if n_rows <= explicit_perm_limit:
            self.perm = torch.randperm(n_rows, generator=self.g, device=device)
            self.affine = None
        else:
            self.perm = None
            pg = torch.Generator().manual_seed(int(seed) + 7919)
            while True:
                a = int(torch.randint(1, min(n_rows, 1 << 31), (1,), generator=pg))
                if math.gcd(a, n_rows) == 1:
                    break
            c = int(torch.randint(0, n_rows, (1,), generator=pg))
            self.affine = (a, c)

    def draw(self, n: int, dtype=torch.int64) -> torch.Tensor:
        u = torch.rand(n, dtype=torch.float64, device=self.device, generator=self.g)
        rank = torch.searchsorted(self.cdf, u).clamp_(max=self.n_rows - 1)
        if self.perm is not None:
            rows = self.perm[rank]
        else:
            a, c = self.affine
            rows = (rank * a + c) % self.n_rows
        return rows.to(dtype)


def bernoulli_lookup_stream(n_rows: int, p: float, seed: int, device="cpu",
                            repeat: float = 1.0, dtype=torch.int64) -> torch.Tensor:
    """A lookup stream whose set of distinct rows is a Bernoulli(p) sample of the table.

    Every selected row appears once, plus ``repeat`` * (number selected) further lookups drawn
    from the selected rows with a skew towards a few hot ones, all in shuffled order (duplicates
    are what a real lookup stream is full of)."""
    g = _gen(seed, device)
    picked = torch.nonzero(torch.rand(n_rows, device=device, generator=g) < p).reshape(-1)
    n_sel = picked.numel()
    n_extra = int(repeat * n_sel)
    if n_sel and n_extra:
        u = torch.rand(n_extra, device=device, generator=g)
        extra = picked[(u * u * u * n_sel).long().clamp_(max=n_sel - 1)]
        stream = torch.cat([picked, extra])
    else:
        stream = picked
    if stream.numel():
        stream = stream[torch.randperm(stream.numel(), device=device, generator=g)]
    return stream.to(dtype)


def lookup_batches(w: Workload, table_index: int, seed: int, device="cpu",
                   n_rows: int | None = None, iterations: int | None = None,
                   dtype=torch.int64):
    """Yields one index tensor per training iteration for one table of workload ``w``
    (``batch * pooling`` lookups each).  ``zipf_until_coverage`` workloads yield rounds for ever:
    the caller stops once the touched fraction it measures reaches ``w.dirty_fraction``."""
    rows = w.n_rows if n_rows is None else n_rows
    s = seed * 1000 + 31 * table_index + 5
    if w.lookups == "bernoulli":
        yield bernoulli_lookup_stream(rows, w.dirty_fraction, s, device, dtype=dtype)
        return
    z = ZipfSampler(rows, w.zipf_s, s, device)
    if w.lookups == "zipf_batches":
        per_iter = w.batch * w.pooling
        for _ in range(w.iterations if iterations is None else iterations):
            yield z.draw(per_iter, dtype)
        return
    if w.lookups == "zipf_until_coverage":
        per_round = max(1024, min(16_000_000, rows // 2))
        n = 0
        while iterations is None or n < iterations:
            yield z.draw(per_round, dtype)
            n += 1
        return
    raise ValueError(w.lookups)


def sample_positions(n: int, fraction: float, seed: int, device="cpu", min_rows: int = 256) -> torch.Tensor:
    """Uniform sample (with replacement, sorted) of positions in [0, n): max(min_rows, fraction * n)
    draws; the input of the greedy-parameter profiling (Section 5.2: 0.001 % of the checkpoint)."""
    m = max(min_rows, int(math.ceil(fraction * n)))
    g = _gen(seed, device)
    return torch.sort((torch.rand(m, dtype=torch.float64, device=device, generator=g) * n).long().clamp_(max=n - 1)).values
