"""CPU oracle for the Check-N-Run checkpoint-encoder path.

TEST INFRASTRUCTURE ONLY: imported by the test-suite, the smoke check and the CPU-baseline leg of
the benchmark.  Nothing in the GPU library imports this package, and this package imports nothing
from the GPU library.
"""
from .cnr_oracle import *  # noqa: F401,F403
from .selection import mean_l2, select_greedy_params, taper_choice  # noqa: F401
