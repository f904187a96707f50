"""CPU oracle for the decision-robustness summary -- TEST INFRASTRUCTURE ONLY.

The paper's closing argument (Section 4 and the conclusion) is that the
deviations between predicted and real behaviour did not change which
technique the models select.  Stated for a batch of decision tables over one
grid, table 0 being the tuning of the parameters as measured and tables
1..n-1 the tunings of perturbed copies of them:

  agree[op][m][P]       how many of the tables 1..n-1 hold the same decision as
                        table 0 in that cell
  max_dev[op][m][P]     the largest abs(T_t - T_0) / T_0 over those tables (T:
                        the predicted time of the cell's winner); 0 for n = 1;
                        a NaN quotient is skipped
  table_agree[t]        in how many cells table t holds the decision of table 0
                        (table_agree[0] = number of cells)

  key_mode 0: decision = strategy id
  key_mode 1: decision = (strategy id, s)

The fraction of perturbed parameter sets that keep a cell's decision is
agree / (n - 1).  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this; the HIP library shares no code with it.
"""
from __future__ import annotations

import numpy as np


def robustness_loops(cells: np.ndarray, key_mode: int):
    """The definition, cell by cell (small inputs only).

    cells: structured array [table][operation][m][P] with fields time, s, strategy.
    Returns (agree uint32 [ops][m][P], max_dev float64 [ops][m][P], table_agree uint32 [tables]).
    """
    if key_mode not in (0, 1):
        raise ValueError("key_mode")
    nt, n_ops, n_m, n_P = cells.shape
    agree = np.zeros((n_ops, n_m, n_P), dtype=np.uint32)
    max_dev = np.zeros((n_ops, n_m, n_P), dtype=np.float64)
    table_agree = np.zeros(nt, dtype=np.uint32)
    table_agree[0] = n_ops * n_m * n_P
    for op in range(n_ops):
        for mi in range(n_m):
            for pi in range(n_P):
                base = cells[0, op, mi, pi]
                for t in range(1, nt):
                    c = cells[t, op, mi, pi]
                    same = int(c["strategy"]) == int(base["strategy"])
                    if key_mode == 1:
                        same = same and int(c["s"]) == int(base["s"])
                    if same:
                        agree[op, mi, pi] += 1
                        table_agree[t] += 1
                    t0 = float(base["time"])
                    with np.errstate(divide="ignore", invalid="ignore"):
                        dev = np.float64(abs(float(c["time"]) - t0)) / np.float64(t0)
                    if dev > max_dev[op, mi, pi]:          # false for NaN
                        max_dev[op, mi, pi] = dev
    return agree, max_dev, table_agree


def robustness(cells: np.ndarray, key_mode: int):
    """The same with array operations (any size the host memory holds)."""
    if key_mode not in (0, 1):
        raise ValueError("key_mode")
    nt = cells.shape[0]
    base = cells[0]
    same = cells["strategy"][1:] == base["strategy"][None]
    if key_mode == 1:
        same &= cells["s"][1:] == base["s"][None]
    agree = same.sum(axis=0, dtype=np.uint32)
    table_agree = np.empty(nt, dtype=np.uint32)
    table_agree[0] = base.size
    table_agree[1:] = same.reshape(nt - 1, base.size).sum(axis=1, dtype=np.uint32)
    with np.errstate(divide="ignore", invalid="ignore"):
        dev = np.abs(cells["time"][1:] - base["time"][None]) / base["time"][None]
    max_dev = np.fmax.reduce(dev, axis=0, initial=0.0) if nt > 1 else np.zeros(base.shape)
    return agree, max_dev.astype(np.float64), table_agree
