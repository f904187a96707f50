"""Pins for the scoring oracle (prediction against measurement, the step after the tuning in
the paper's Section 4): values fixed by hand and by arithmetic that is exact, the two error
modes the paper reports (a constant offset; a delay of the small messages), an independent
array evaluation of the verdicts, and invariants."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from plogp_workloads import make_workload
from tests.helpers import rounded_model

# g(z) = 32 + z / 8 on powers of two, L = 64: every model value is an integer (exact in binary64)
X = np.array([1, 8, 64, 512, 4096, 32768], dtype=np.float64)
Y = 32.0 + X / 8.0
LAT = 64.0
ALL = 0x1FFF


def closed_form(sid, m, P, s):
    """Integer closed forms of Tables 1 and 2 on the affine table above."""
    g = lambda z: Fraction(32) + Fraction(z, 8)
    q, fl, cl = P - 1, P.bit_length() - 1, (P - 1).bit_length()
    R = 2 * g(1) + 3 * LAT
    k = -(-m // s) if s else 0
    return {
        0: q * g(m) + LAT, 1: q * g(m) + R, 2: q * g(s) * k + LAT if s else None,
        3: q * (g(m) + LAT), 4: q * (g(m) + R),
        5: q * (g(s) + LAT) + g(s) * (k - 1) if s else None,
        6: cl * (2 * g(m) + LAT), 7: fl * g(m) + cl * LAT, 8: fl * g(m) + cl * R,
        9: fl * g(s) * k + cl * LAT if s else None,
        10: q * g(m) + LAT, 11: sum(g(j * m) for j in range(1, P)) + q * LAT,
        12: sum(g((1 << j) * m) for j in range(cl)) + cl * LAT,
    }[sid]


def grid():
    m = np.array([8, 64, 200 * 8, 4096], dtype=np.uint64)
    P = np.array([2, 3, 4, 7, 8, 33], dtype=np.uint32)
    seg = np.empty((13, m.size, P.size), dtype=np.uint32)
    seg[:] = np.array([8, 16, 64, 512], dtype=np.uint32)[None, :, None]
    return m, P, seg


def test_predictions_equal_the_integer_closed_forms_and_a_perfect_measurement_scores_zero():
    m, P, seg = grid()
    want = np.array([[[float(closed_form(sid, int(mm), int(pp), int(seg[sid, i, j])))
                       for j, pp in enumerate(P)] for i, mm in enumerate(m)] for sid in range(13)])
    pred, verdict, score = oracle.score_grid(X, Y, LAT, m, P, ALL, want, seg)
    assert (pred == want).all()
    assert (score["sum_abs_err"] == 0).all() and (score["max_abs_err"] == 0).all()
    assert (score["count"] == m.size * P.size).all()
    assert (verdict["regret"] == 0).all()
    assert (verdict["pred_best"] == verdict["meas_best"]).all()
    # the verdicts from plain array operations (first minimum = lowest id)
    assert (verdict["pred_best"][0] == np.argmin(want[:10], axis=0)).all()
    assert (verdict["pred_best"][1] == 10 + np.argmin(want[10:], axis=0)).all()


def test_hand_written_cell():
    # one cell, two Broadcast strategies: flat tree (id 0) and chain (id 3), m = 64, P = 4:
    # flat 3 * 40 + 64 = 184, chain 3 * (40 + 64) = 312.  Measured 400 and 300: the model picks
    # the flat tree, the measurement the chain; regret 400 / 300 - 1; errors 216/400 and 12/300.
    m = np.array([64], dtype=np.uint64)
    P = np.array([4], dtype=np.uint32)
    mask = (1 << 0) | (1 << 3)
    meas = np.array([[[400.0]], [[300.0]]])
    pred, verdict, score = oracle.score_grid(X, Y, LAT, m, P, mask, meas, np.zeros((2, 1, 1), np.uint32))
    assert pred.ravel().tolist() == [184.0, 312.0]
    assert verdict.shape == (1, 1, 1)
    assert (int(verdict["pred_best"][0, 0, 0]), int(verdict["meas_best"][0, 0, 0])) == (0, 3)
    assert verdict["regret"][0, 0, 0] == 400.0 / 300.0 - 1.0
    assert score["sum_abs_err"].tolist() == [216.0 / 400.0, 12.0 / 300.0]
    assert score["max_abs_err"].tolist() == [216.0 / 400.0, 12.0 / 300.0]
    assert score["count"].tolist() == [1, 1]


def test_constant_offset_keeps_every_decision():
    # the first error mode of the paper's measurements: every curve is shifted by the same
    # constant, which moves the errors but cannot change which strategy is fastest
    m, P, seg = grid()
    pred, _, _ = oracle.score_grid(X, Y, LAT, m, P, ALL, np.ones((13, m.size, P.size)), seg)
    meas = pred + 1024.0                      # exact: integers
    _, verdict, score = oracle.score_grid(X, Y, LAT, m, P, ALL, meas, seg)
    assert (verdict["pred_best"] == verdict["meas_best"]).all() and (verdict["regret"] == 0).all()
    assert (score["max_abs_err"] > 0).all()
    e = np.abs((pred - meas) / meas)
    assert np.allclose(score["sum_abs_err"], e.sum(axis=(1, 2)), rtol=1e-13, atol=0)
    assert (score["max_abs_err"] == e.max(axis=(1, 2))).all()


def test_small_message_delay_can_flip_a_decision_and_the_regret_says_by_how_much():
    # the second error mode: the strategy the model prefers for the smallest size is measured
    # twice as slow there; the verdict of exactly those cells changes
    m, P, seg = grid()
    pred, v0, _ = oracle.score_grid(X, Y, LAT, m, P, ALL, np.ones((13, m.size, P.size)), seg)
    meas = pred.copy()
    for pj in range(P.size):
        meas[v0["pred_best"][0, 0, pj], 0, pj] *= 4.0
    _, verdict, _ = oracle.score_grid(X, Y, LAT, m, P, ALL, meas, seg)
    b = verdict[0]
    assert (b["pred_best"][1:] == b["meas_best"][1:]).all() and (b["regret"][1:] == 0).all()
    for pj in range(P.size):
        col = meas[:10, 0, pj]
        assert b["meas_best"][0, pj] == np.argmin(col)
        assert b["regret"][0, pj] == col[b["pred_best"][0, pj]] / col.min() - 1.0
        assert b["regret"][0, pj] > 0
    assert (verdict[1]["regret"] == 0).all()           # the Scatter plane is untouched


def test_every_rounding_of_the_predictions_on_a_config_table():
    # on a table that is not exact in binary64: the prediction equals the correctly rounded
    # replay of each operation in rational arithmetic
    wl = make_workload(1)
    x, y, L = wl.sizes[0], wl.gaps[0], float(wl.L[0])
    m = wl.m[[0, 20, 41, 63]]
    P = np.array([2, 5, 16, 50], dtype=np.uint32)
    seg = np.empty((13, 4, 4), dtype=np.uint32)
    seg[:] = np.minimum(m, 1024).astype(np.uint32)[None, :, None]
    pred, _, _ = oracle.score_grid(x, y, L, m, P, ALL, np.ones((13, 4, 4)), seg)
    for sid in range(13):
        for i in range(4):
            for j in range(4):
                s = int(seg[sid, i, j]) if sid in (2, 5, 9) else 0
                assert pred[sid, i, j] == rounded_model(x, y, L, sid, int(m[i]), int(P[j]), s)


def test_sum_order_rows_first_and_operation_planes():
    rng = np.random.default_rng(4)
    m, P, seg = grid()
    mask = (1 << 10) | (1 << 11) | (1 << 12)              # Scatter only: one plane
    meas = 50.0 + 1000.0 * rng.random((3, m.size, P.size))
    pred, verdict, score = oracle.score_grid(X, Y, LAT, m, P, mask, meas, seg[:3])
    assert verdict.shape == (1, m.size, P.size)
    assert set(np.unique(verdict["pred_best"])) <= {10, 11, 12}
    e = np.abs((pred - meas) / meas)
    for r in range(3):
        total = 0.0
        for i in range(m.size):
            row = 0.0
            for j in range(P.size):
                row = row + e[r, i, j]
            total = total + row
        assert score["sum_abs_err"][r] == total
    assert (verdict["meas_best"][0] == 10 + np.argmin(meas, axis=0)).all()


def test_bad_arguments():
    m, P, seg = grid()
    meas = np.ones((13, m.size, P.size))
    bad = seg.copy()
    bad[5, 0, 0] = 16                                       # s above m = 8
    with pytest.raises(ValueError):
        oracle.score_grid(X, Y, LAT, m, P, ALL, meas, bad)
    with pytest.raises(ValueError):
        oracle.score_grid(X, Y, LAT, m, np.array([1], dtype=np.uint32), 1, meas[:1, :, :1], seg[:1, :, :1])
