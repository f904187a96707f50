"""Seeded synthetic pLogP tables and tuning grids.

This module only *makes inputs*: measured-looking gap tables (sizes, gaps, L)
and the (m, P, s) grids that are swept.  It holds none of the method's
arithmetic (no interpolation, no cost model, no arg-min), so the CPU oracle,
the HIP library, the tests and the benchmark can all draw their inputs from
it without sharing any code of the method itself.

The paper's only workload is one measured parameter table of a 50-node,
100 Mbit/s Ethernet cluster (Section 2); that table is not printed in the
paper, so seeded synthetic tables of the same shape stand in for it.
Units: bytes for sizes, microseconds for gaps and latency.
"""
from .configs import (  # noqa: F401
    Workload,
    SplitMix64,
    make_workload,
    make_measurements,
    make_perturbed,
    log_spaced_sizes,
    STRATEGY_NAMES,
    BCAST_IDS,
    SCATTER_IDS,
    SEGMENTED_IDS,
    ALL_STRATEGIES_MASK,
    NO_CAP,
)
