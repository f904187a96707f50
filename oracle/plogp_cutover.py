"""CPU oracle for the cut-over extraction -- TEST INFRASTRUCTURE ONLY.

The tuned decisions are used as thresholds along the message size: below some
size one technique (or no segmentation) is predicted fastest, above it another
(paper, Section 3.1, the closing remark on how the chosen segment size is
applied, and Section 1, the choice per pattern, message size and node count).
This module states that compression in the plainest way: one row of the
decision table is the sequence of cells of one (table, operation, P) read along
the grid's message sizes in their given order; a run starts at the first cell
and at every cell whose key differs from the key of the cell before it.

  key_mode 0: key = strategy id            (which technique)
  key_mode 1: key = (strategy id, s)       (which technique and segment size)

A run is reported as (m_from, s, strategy): the message size of its first
cell and that cell's s and strategy.  Rows are ordered (table, operation, P);
row_offsets[r] .. row_offsets[r+1] are the runs of row r.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this; the HIP library shares no code with it.
"""
from __future__ import annotations

import numpy as np

RUN_DTYPE = np.dtype([("m_from", "<u8"), ("s", "<u4"), ("strategy", "<u4")])


def _key(cell, key_mode):
    return (int(cell["strategy"]),) if key_mode == 0 else (int(cell["strategy"]), int(cell["s"]))


def cutovers_loops(cells: np.ndarray, m: np.ndarray, key_mode: int):
    """The definition, cell by cell (small inputs only).

    cells: structured array [table][operation][m][P] with fields s, strategy.
    Returns (row_offsets uint64[n_rows + 1], runs RUN_DTYPE[n_runs]).
    """
    if key_mode not in (0, 1):
        raise ValueError("key_mode")
    nt, n_ops, n_m, n_P = cells.shape
    offsets = [0]
    runs = []
    for t in range(nt):
        for op in range(n_ops):
            for pi in range(n_P):
                prev = None
                for mi in range(n_m):
                    c = cells[t, op, mi, pi]
                    k = _key(c, key_mode)
                    if mi == 0 or k != prev:
                        runs.append((int(m[mi]), int(c["s"]), int(c["strategy"])))
                    prev = k
                offsets.append(len(runs))
    return np.asarray(offsets, dtype=np.uint64), np.asarray(runs, dtype=RUN_DTYPE).reshape(-1)


def cutovers(cells: np.ndarray, m: np.ndarray, key_mode: int):
    """The same with array operations (any size the host memory holds)."""
    if key_mode not in (0, 1):
        raise ValueError("key_mode")
    nt, n_ops, n_m, n_P = cells.shape
    strat = cells["strategy"]
    seg = cells["s"]
    starts = np.ones(cells.shape, dtype=bool)              # the first cell of a row starts a run
    if n_m > 1:
        differs = strat[:, :, 1:, :] != strat[:, :, :-1, :]
        if key_mode == 1:
            differs |= seg[:, :, 1:, :] != seg[:, :, :-1, :]
        starts[:, :, 1:, :] = differs
    by_row = np.ascontiguousarray(np.transpose(starts, (0, 1, 3, 2)))   # [table][op][P][m]
    counts = by_row.reshape(-1, n_m).sum(axis=1, dtype=np.uint64) if n_m else np.zeros(nt * n_ops * n_P, np.uint64)
    offsets = np.zeros(counts.size + 1, dtype=np.uint64)
    np.cumsum(counts, out=offsets[1:])
    t_i, op_i, p_i, m_i = np.nonzero(by_row)               # row-major: rows in order, m ascending
    runs = np.empty(t_i.size, dtype=RUN_DTYPE)
    runs["m_from"] = np.asarray(m, dtype=np.uint64)[m_i]
    runs["s"] = seg[t_i, op_i, m_i, p_i]
    runs["strategy"] = strat[t_i, op_i, m_i, p_i]
    return offsets, runs


def expand(row_offsets: np.ndarray, runs: np.ndarray, m: np.ndarray, shape):
    """Inverse for key_mode 0/1 checks: the strategy of every cell from the runs.

    Needs the grid's sizes to be free of repeats inside a row's run starts, so it
    locates a run by counting: runs of a row are laid down in order and each
    lasts until the next one's first cell index, found by matching m_from from
    the previous start onwards.
    """
    nt, n_ops, n_m, n_P = shape
    out = np.empty(shape, dtype=np.uint32)
    r = 0
    for t in range(nt):
        for op in range(n_ops):
            for pi in range(n_P):
                lo, hi = int(row_offsets[r]), int(row_offsets[r + 1])
                pos = 0
                for k in range(lo, hi):
                    # first index >= pos whose size equals this run's m_from
                    start = pos
                    while int(m[start]) != int(runs["m_from"][k]):
                        start += 1
                    if k > lo:
                        out[t, op, pos_prev:start, pi] = runs["strategy"][k - 1]
                    pos_prev = start
                    pos = start + 1
                out[t, op, pos_prev:, pi] = runs["strategy"][hi - 1]
                r += 1
    return out
