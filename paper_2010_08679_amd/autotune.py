"""Automatic choice of the greedy search parameters by profiling a small sample of the checkpoint
(Section 5.2, "Parameter selection").

Plumbing only: the library's ``cnr_select_greedy_params`` quantizes the sample over the grids,
computes the mean l2 errors and makes the choice (its header states the reading taken for "tapers
off"); this module allocates the scratch buffer it needs and names the entries of its report.
"""
from __future__ import annotations

import torch

from . import binding as B

DEFAULT_BINS = (5, 10, 15, 20, 25, 30, 35, 40, 45, 50)
DEFAULT_RATIOS = (0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 1.0)


def select_greedy_params(ctx, table: torch.Tensor, n_rows: int, dim: int, sample_ids: torch.Tensor,
                         bits: int, bins_grid=DEFAULT_BINS, ratio_grid=DEFAULT_RATIOS,
                         taper: float = 0.05, stream=None):
    """Returns ((num_bins, ratio), report) for the rows ``sample_ids`` (uint32 bits in an int32
    tensor) of ``table``; report maps "naive", ("bins", nb) and ("ratio", r) to mean l2 errors."""
    need = B.cnr_select_scratch_bytes(sample_ids.numel(), dim, bits)
    scratch = torch.empty((need + 7) // 8, dtype=torch.int64, device=table.device)
    chosen, values = B.cnr_select_greedy_params(ctx, table, n_rows, dim, sample_ids, bits, bins_grid, ratio_grid,
                                                taper, scratch, stream)
    keys = ["naive"] + [("bins", nb) for nb in bins_grid] + [("ratio", r) for r in ratio_grid]
    return chosen, dict(zip(keys, values))
