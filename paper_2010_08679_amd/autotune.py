"""Automatic choice of the greedy search parameters by profiling a small sample of the checkpoint
(Section 5.2, "Parameter selection").

The method estimates the mean l2 error from a uniform sample of the checkpoint's rows (0.001 % by
default), quantizes that sample with a grid of parameter values, and keeps the value at which the
improvement over naive asymmetric quantization tapers off.  Every quantization and every error runs
in libcnr's kernels (``cnr_quantize_rows``, ``cnr_quant_error``); only the comparison of a dozen
means happens here on the host.

Reading of "tapers off" (the paper gives no threshold): with I(p) = 1 - E(p) / E_naive the
improvement at parameter value p, the choice is the smallest p of the grid whose improvement is
within ``taper`` (relative, 5 % by default) of the best improvement on the grid.  num_bins is chosen
first at ratio 1, then the ratio with that num_bins, as in the paper's figures.
"""
from __future__ import annotations

import torch

from . import binding as B

DEFAULT_BINS = (5, 10, 15, 20, 25, 30, 35, 40, 45, 50)
DEFAULT_RATIOS = (0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 1.0)


def _taper_choice(grid, errors, e_naive, taper):
    gains = [1.0 - e / e_naive if e_naive > 0 else 0.0 for e in errors]
    best = max(gains)
    if best <= 0.0:
        return grid[0]
    for p, g in zip(grid, gains):
        if g >= (1.0 - taper) * best:
            return p
    return grid[-1]


def select_greedy_params(ctx, table: torch.Tensor, n_rows: int, dim: int, sample_ids: torch.Tensor,
                         bits: int, bins_grid=DEFAULT_BINS, ratio_grid=DEFAULT_RATIOS,
                         taper: float = 0.05, stream=None):
    """Returns ((num_bins, ratio), report) for the rows ``sample_ids`` (uint32 bits in an int32
    tensor) of ``table``; report maps "naive", ("bins", nb) and ("ratio", r) to mean l2 errors."""
    m = sample_ids.numel()
    dev = table.device
    scale = torch.empty(m, dtype=torch.float32, device=dev)
    bias = torch.empty(m, dtype=torch.float32, device=dev)
    packed = torch.empty(m * B.cnr_packed_row_bytes(dim, bits), dtype=torch.uint8, device=dev)
    err = torch.empty(m, dtype=torch.float64, device=dev)
    mean = torch.zeros(1, dtype=torch.float64, device=dev)

    def mean_error(mode, greedy):
        B.cnr_quantize_rows(ctx, table, n_rows, dim, sample_ids, None, m, bits, mode, greedy, scale, bias,
                            packed=packed, stream=stream)
        B.cnr_quant_error(ctx, table, n_rows, dim, sample_ids, None, m, bits, packed, scale, bias, err, mean,
                          stream=stream)
        return float(mean.item())

    report = {"naive": mean_error(B.CNR_RANGE_MINMAX, None)}
    for nb in bins_grid:
        report[("bins", nb)] = mean_error(B.CNR_RANGE_GREEDY, (nb, 1.0))
    num_bins = _taper_choice(list(bins_grid), [report[("bins", nb)] for nb in bins_grid], report["naive"], taper)
    for r in ratio_grid:
        report[("ratio", r)] = mean_error(B.CNR_RANGE_GREEDY, (num_bins, r))
    ratio = _taper_choice(list(ratio_grid), [report[("ratio", r)] for r in ratio_grid], report["naive"], taper)
    return (num_bins, ratio), report
