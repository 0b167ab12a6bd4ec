"""Greedy-parameter selection by profiling (Section 5.2, "Parameter selection"), CPU reference.

TEST INFRASTRUCTURE ONLY.  The paper samples a small fraction of the checkpoint uniformly (0.001 %
by default), quantizes the sample with different parameter values, computes the mean l2 errors and
keeps the value at which the improvement tapers off.  The sample is an input here (the caller draws
it); quantization and errors come from the C oracle.

Reading taken for "tapers off" (no threshold is given): with I(p) = 1 - E(p) / E_naive, the value
kept is the smallest p of the grid whose improvement is within `taper` (relative) of the largest
improvement on the grid.  num_bins is chosen first at ratio 1, then the ratio at that num_bins, the
order of the paper's two figures.
"""
from __future__ import annotations

import numpy as np

from . import cnr_oracle as C


def taper_choice(grid, errors, naive, taper):
    improvement = [1.0 - e / naive if naive > 0 else 0.0 for e in errors]
    top = max(improvement)
    if top <= 0.0:
        return grid[0]
    return next(p for p, g in zip(grid, improvement) if g >= (1.0 - taper) * top)


def mean_l2(rows: np.ndarray, bits: int, mode: int, num_bins: int = 0, ratio: float = 1.0,
            n_threads: int = 1) -> float:
    q = C.quantize_rows(rows, None, bits, mode=mode, num_bins=num_bins, ratio=ratio, n_threads=n_threads)
    return C.row_l2(rows, C.dequantize(q["codes"], q["scale"], q["bias"]))[1]


def select_greedy_params(rows: np.ndarray, bits: int, bins_grid, ratio_grid, taper: float = 0.05,
                         n_threads: int = 1):
    """Returns ((num_bins, ratio), report) for the sampled ``rows`` [m, dim]; report maps "naive",
    ("bins", nb) and ("ratio", r) to mean l2 errors."""
    report = {"naive": mean_l2(rows, bits, C.RANGE_MINMAX, n_threads=n_threads)}
    for nb in bins_grid:
        report[("bins", nb)] = mean_l2(rows, bits, C.RANGE_GREEDY, nb, 1.0, n_threads)
    num_bins = taper_choice(list(bins_grid), [report[("bins", nb)] for nb in bins_grid], report["naive"], taper)
    for r in ratio_grid:
        report[("ratio", r)] = mean_l2(rows, bits, C.RANGE_GREEDY, num_bins, r, n_threads)
    ratio = taper_choice(list(ratio_grid), [report[("ratio", r)] for r in ratio_grid], report["naive"], taper)
    return (num_bins, ratio), report
