"""Pins of the robustness oracle (how many perturbed tunings keep a cell's decision,
paper Section 4 / conclusion): a hand-written table, the definition cell by cell
against the array form, invariants that a wrong axis, a dropped table 0 or a
swapped key would break, and the end-to-end facts that the tuning oracle fixes."""
import numpy as np
import pytest

import oracle
from oracle import plogp_robust as orb
from plogp_workloads import make_perturbed, make_workload


def table(entries):
    """[tables][1][m][P] from nested lists of (time, s, strategy)."""
    a = np.array(entries, dtype=object)
    nt, n_m, n_P = a.shape[:3]
    cells = np.zeros((nt, 1, n_m, n_P), dtype=oracle.CELL_DTYPE)
    for t in range(nt):
        for mi in range(n_m):
            for pi in range(n_P):
                cells[t, 0, mi, pi] = tuple(a[t, mi, pi])
    return cells


def test_hand_written_table():
    # 3 tables, 2 sizes, 2 process counts; table 0 is the reference
    cells = table([
        [[(10.0, 0, 3), (20.0, 64, 5)], [(40.0, 0, 7), (80.0, 128, 9)]],
        [[(11.0, 0, 3), (25.0, 32, 5)], [(30.0, 0, 6), (80.0, 128, 9)]],
        [[(9.0, 0, 4), (20.0, 64, 5)], [(44.0, 0, 7), (100.0, 128, 2)]],
    ])
    for fn in (orb.robustness_loops, orb.robustness):
        agree, dev, per_table = fn(cells, 0)
        assert agree[0].tolist() == [[1, 2], [1, 1]]
        assert per_table.tolist() == [4, 3, 2]
        assert dev[0].tolist() == [[0.1, 0.25], [0.25, 0.25]]
        agree, dev, per_table = fn(cells, 1)
        assert agree[0].tolist() == [[1, 1], [1, 1]]     # table 1 changed s in cell (0, 1)
        assert per_table.tolist() == [4, 2, 2]


def random_cells(rng, nt, n_ops, n_m, n_P, p_same):
    cells = np.zeros((nt, n_ops, n_m, n_P), dtype=oracle.CELL_DTYPE)
    cells["strategy"] = rng.integers(0, 13, size=cells.shape)
    cells["s"] = rng.integers(0, 3, size=cells.shape) * 8
    cells["time"] = rng.random(cells.shape) * 100 + 1
    keep = rng.random(cells.shape) < p_same
    for name in ("strategy", "s"):
        cells[name] = np.where(keep, cells[name][:1], cells[name])
    return cells


@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (2, 1, 3, 5), (7, 2, 9, 4), (30, 2, 5, 11)])
@pytest.mark.parametrize("key_mode", [0, 1])
def test_loops_against_arrays(shape, key_mode):
    cells = random_cells(np.random.default_rng(sum(shape)), *shape, p_same=0.6)
    a1, d1, t1 = orb.robustness_loops(cells, key_mode)
    a2, d2, t2 = orb.robustness(cells, key_mode)
    assert (a1 == a2).all() and (t1 == t2).all()
    assert (d1.view(np.uint64) == d2.view(np.uint64)).all()
    assert a1.dtype == np.uint32 and t1.dtype == np.uint32 and d1.dtype == np.float64


def test_invariants():
    rng = np.random.default_rng(5)
    cells = random_cells(rng, 12, 2, 6, 7, p_same=0.7)
    a0, d0, t0 = orb.robustness(cells, 0)
    a1, d1, t1 = orb.robustness(cells, 1)
    n_cells = cells[0].size
    assert (a1 <= a0).all() and (a0 <= 11).all()              # a stricter key agrees less often
    assert int(a0.sum()) == int(t0[1:].sum()) and int(a1.sum()) == int(t1[1:].sum())
    assert t0[0] == n_cells and (t0 <= n_cells).all()
    assert (d0 == d1).all()                                     # the deviation ignores the key
    # the order of the perturbed tables does not matter per cell; it permutes table_agree
    perm = np.concatenate([[0], 1 + rng.permutation(11)])
    a2, d2, t2 = orb.robustness(cells[perm], 1)
    assert (a2 == a1).all() and (d2 == d1).all() and (t2 == t1[perm]).all()
    # table 0 is the reference: swapping it with another table changes the counts
    swapped = cells.copy()
    swapped[[0, 1]] = swapped[[1, 0]]
    assert not (orb.robustness(swapped, 1)[0] == a1).all()
    # copies of table 0 agree everywhere and deviate nowhere
    same = np.repeat(cells[:1], 5, axis=0)
    a, d, t = orb.robustness(same, 1)
    assert (a == 4).all() and (d == 0).all() and (t == n_cells).all()
    # the deviation is relative to table 0, not to the other table
    two = cells[:2].copy()
    two["time"][0], two["time"][1] = 4.0, 5.0
    assert (orb.robustness(two, 0)[1] == 0.25).all()
    two["time"][0], two["time"][1] = 5.0, 4.0
    assert (orb.robustness(two, 0)[1] == 0.2).all()


def test_degenerate_times():
    cells = np.zeros((3, 1, 1, 2), dtype=oracle.CELL_DTYPE)
    cells["time"][:, 0, 0, 0] = [0.0, 0.0, 0.0]          # 0 / 0: skipped
    cells["time"][:, 0, 0, 1] = [0.0, 1.0, 2.0]          # x / 0: infinite
    for fn in (orb.robustness_loops, orb.robustness):
        _, d, _ = fn(cells, 0)
        assert d[0, 0, 0] == 0.0 and np.isinf(d[0, 0, 1])
    with pytest.raises(ValueError):
        orb.robustness(cells, 2)


def test_unperturbed_copies_of_a_real_tuning_agree_and_perturbed_ones_partly():
    base = make_workload(1)
    same = make_perturbed(base, 6, 0.0)
    assert same.n_tables == 7 and (same.gaps == base.gaps[0]).all() and (same.L == base.L[0]).all()
    cells, _ = oracle.tune_workload(same)
    a, d, t = orb.robustness(cells, 1)
    assert (a == 6).all() and (d == 0).all()
    wl = make_perturbed(base, 40, 0.2, seed=3)
    assert (wl.sizes == base.sizes[0]).all()
    ratio = wl.gaps[1:] / base.gaps[0]
    assert ratio.min() >= 0.8 and ratio.max() <= 1.2 and ratio.std() > 0.05
    assert (np.abs(wl.L[1:] / base.L[0] - 1) <= 0.2).all() and wl.L[1:].std() > 0
    cells, _ = oracle.tune_workload(wl)
    a, d, t = orb.robustness(cells, 1)
    frac = a / 40.0
    # 20 % noise moves some decisions, most cells keep theirs; predicted times move by at most
    # about the noise (every model is a positive combination of gaps and L)
    assert 0.3 < frac.mean() < 1.0 and frac.min() < 1.0
    assert 0.0 < d.max() <= 0.2 * (1 + 1e-9) / (1 - 0.2) + 0.2
    a0, _, _ = orb.robustness(cells, 0)
    assert (a0 >= a).all() and a0.sum() > a.sum()
