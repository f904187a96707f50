"""Pins for the cut-over oracle: hand-written rows, the two implementations
against each other, invariants (paper, Section 3.1: the decisions are used as
thresholds along the message size)."""
import numpy as np
import pytest

from oracle import CELL_DTYPE
from oracle import plogp_cutover as oc


def table_from(ids, ss):
    """cells[1][1][m][P] from per-P columns of ids and s along m."""
    ids = np.asarray(ids, dtype=np.uint32)      # [P][m]
    ss = np.asarray(ss, dtype=np.uint32)
    n_P, n_m = ids.shape
    cells = np.zeros((1, 1, n_m, n_P), dtype=CELL_DTYPE)
    cells["strategy"][0, 0] = ids.T
    cells["s"][0, 0] = ss.T
    cells["time"] = 1.0
    return cells


M = np.array([8, 16, 32, 64, 128, 256], dtype=np.uint64)


def test_hand_written_row_by_strategy():
    # one P: flat tree for small sizes, segmented chain from 64 bytes on (s changes inside)
    cells = table_from([[0, 0, 0, 5, 5, 5]], [[0, 0, 0, 32, 64, 64]])
    for fn in (oc.cutovers_loops, oc.cutovers):
        off, runs = fn(cells, M, 0)
        assert off.tolist() == [0, 2]
        assert runs.tolist() == [(8, 0, 0), (64, 32, 5)]


def test_hand_written_row_by_strategy_and_segment():
    cells = table_from([[0, 0, 0, 5, 5, 5]], [[0, 0, 0, 32, 64, 64]])
    for fn in (oc.cutovers_loops, oc.cutovers):
        off, runs = fn(cells, M, 1)
        assert off.tolist() == [0, 3]
        assert runs.tolist() == [(8, 0, 0), (64, 32, 5), (128, 64, 5)]


def test_rows_are_ordered_table_operation_P_and_a_return_to_an_old_key_is_a_new_run():
    ids = [[7, 7, 9, 9, 7, 7],        # P index 0: back to 7 at the end -> three runs
           [3, 3, 3, 3, 3, 3]]        # P index 1: one run
    ss = [[0, 0, 16, 16, 0, 0], [0] * 6]
    cells = table_from(ids, ss)
    two_ops = np.concatenate([cells, cells], axis=1)
    two_ops["strategy"][0, 1, :, :] = 10          # second plane: a single technique everywhere
    two_ops["s"][0, 1, :, :] = 0
    for fn in (oc.cutovers_loops, oc.cutovers):
        off, runs = fn(two_ops, M, 0)
        assert off.tolist() == [0, 3, 4, 5, 6]
        assert runs.tolist() == [(8, 0, 7), (32, 16, 9), (128, 0, 7), (8, 0, 3), (8, 0, 10), (8, 0, 10)]


def test_single_size_and_constant_rows():
    cells = table_from([[4], [2]], [[0], [8]])
    off, runs = oc.cutovers(cells, M[:1], 1)
    assert off.tolist() == [0, 1, 2]
    assert runs.tolist() == [(8, 0, 4), (8, 8, 2)]


def test_repeated_sizes_are_compared_by_position():
    m = np.array([8, 8, 8, 16], dtype=np.uint64)
    cells = table_from([[0, 3, 3, 0]], [[0, 0, 0, 0]])
    off, runs = oc.cutovers(cells, m, 0)
    assert runs.tolist() == [(8, 0, 0), (8, 0, 3), (16, 0, 0)]


@pytest.mark.parametrize("key_mode", [0, 1])
def test_array_form_equals_the_cell_by_cell_definition(key_mode):
    rng = np.random.default_rng(5)
    nt, n_ops, n_m, n_P = 3, 2, 37, 11
    cells = np.zeros((nt, n_ops, n_m, n_P), dtype=CELL_DTYPE)
    # long runs with occasional changes, like a decision table
    base = rng.integers(0, 4, size=(nt, n_ops, 1, n_P))
    steps = (rng.random((nt, n_ops, n_m, n_P)) < 0.15).cumsum(axis=2)
    cells["strategy"] = (base + steps) % 5
    cells["s"] = 8 * ((rng.random((nt, n_ops, n_m, n_P)) < 0.1).cumsum(axis=2) % 3)
    m = np.sort(rng.integers(1, 1000, size=n_m)).astype(np.uint64) * 8
    a = oc.cutovers_loops(cells, m, key_mode)
    b = oc.cutovers(cells, m, key_mode)
    assert np.array_equal(a[0], b[0])
    assert np.array_equal(a[1], b[1])
    # invariants: one run per row at least, count = changes + 1, first run starts at m[0]
    counts = np.diff(a[0].astype(np.int64))
    assert counts.min() >= 1 and a[0][-1] == a[1].size
    assert np.all(a[1]["m_from"][a[0][:-1].astype(np.int64)] == m[0])


def test_runs_rebuild_the_strategy_plane():
    rng = np.random.default_rng(9)
    shape = (2, 2, 29, 7)
    cells = np.zeros(shape, dtype=CELL_DTYPE)
    cells["strategy"] = (rng.random(shape) < 0.2).cumsum(axis=2) % 6
    m = (np.arange(1, 30, dtype=np.uint64)) * 8          # strictly ascending
    off, runs = oc.cutovers(cells, m, 0)
    assert np.array_equal(oc.expand(off, runs, m, shape), cells["strategy"])


def test_config1_cutovers_match_the_stored_fixture():
    import os
    import oracle
    from plogp_workloads import make_workload
    wl = make_workload(1)
    out, _ = oracle.tune_workload(wl)
    off, runs = oc.cutovers(out, wl.m, 0)
    want = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "cfg1_cutovers.txt")) as f:
        for line in f:
            if line.startswith("#"):
                continue
            P, m_from, strat, s = (int(v) for v in line.split())
            want.setdefault(P, []).append((m_from, s, strat))
    assert sorted(want) == [2, 3, 4, 8, 16, 32, 50]
    for P, rows in want.items():
        pi = int(np.nonzero(wl.P == P)[0][0])
        got = runs[int(off[pi]):int(off[pi + 1])].tolist()
        assert got == rows
    # from four nodes on, large messages go to the segmented chain and small ones do not
    for P, rows in want.items():
        if P >= 4:
            assert rows[-1][2] == 5 and rows[0][2] != 5
