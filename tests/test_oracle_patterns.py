"""Pins of the rows beyond Tables 1 and 2: Gather (ids 13..15) and Barrier (ids 16, 17),
the patterns Section 3 names as built like Broadcast and Scatter.  The paper prints no row
for them, so each is derived here from the pLogP rules and pinned three ways: the event
simulator replays its schedule (who sends what to whom; it knows no closed form), exact
tables give integer closed forms, and the structure ties it to rows the paper does print
(a Gather is its Scatter with every message reversed: the same value bit for bit; a
Barrier is a one-byte fan-in plus a one-byte fan-out: twice a row of Table 1 at g(1))."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import plogp_sim
from plogp_workloads import make_workload
from tests.helpers import F, bits, clog2, exact_g, flog2, rn, rounded_g

X = np.array([1.0, 8.0, 64.0, 500.0, 4096.0, 20000.0, 131072.0, 1048576.0])
Y = np.array([3.0, 3.5, 5.0, 9.0, 40.0, 170.0, 1100.0, 8000.0])
LAT = 7.25
REL = 4e-15


def g_exact(z):
    return exact_g(X, Y, z)


def close(a, b, rel=REL):
    return abs(F(a) - b) <= rel * abs(b)


@pytest.mark.parametrize("sid", [13, 14, 16])
def test_flat_and_chain_rows_equal_the_replay_for_every_P(sid):
    for P in range(2, 17):
        for m in (8, 4096, 70000):
            sim = plogp_sim.completion_time(sid, P, m, 0, g_exact, LAT)
            got = oracle.eval_strategy(X, Y, LAT, sid, m, P)
            assert close(got, sim), (sid, P, m, got, float(sim))


@pytest.mark.parametrize("sid", [15, 17])
def test_binomial_rows_equal_the_replay_at_powers_of_two(sid):
    for P in (2, 4, 8, 16):
        for m in (8, 4096, 20000):
            sim = plogp_sim.completion_time(sid, P, m, 0, g_exact, LAT)
            got = oracle.eval_strategy(X, Y, LAT, sid, m, P)
            assert close(got, sim), (sid, P, m, got, float(sim))


def test_receiving_end_of_the_simulator_on_hand_computed_cases():
    g10 = lambda z: Fraction(10)
    # three nodes send to node 0 at time 0 (g = 10, L = 3): taken in at 13, 23, 33
    progs = {0: [("recv", 1, "a"), ("recv", 2, "a"), ("recv", 3, "a")],
             1: [("send", 0, 8, "a")], 2: [("send", 0, 8, "a")], 3: [("send", 0, 8, "a")]}
    assert plogp_sim.run(progs, g10, Fraction(3)) == 33
    # receptions that arrive more than a gap apart are not delayed: 13, then 40 + 13
    progs = {0: [("recv", 1, "a"), ("recv", 2, "a")],
             1: [("send", 0, 8, "a")],
             2: [("send", 3, 8, "x"), ("send", 3, 8, "y"), ("send", 3, 8, "z"), ("send", 3, 8, "w"), ("send", 0, 8, "a")],
             3: [("recv", 2, "x"), ("recv", 2, "y"), ("recv", 2, "z"), ("recv", 2, "w")]}
    assert plogp_sim.run(progs, g10, Fraction(3)) == 53
    # flat gather of 5 nodes = (P - 1) g + L; flat barrier = twice that
    assert plogp_sim.completion_time(13, 5, 8, 0, g10, 3) == 43
    assert plogp_sim.completion_time(16, 5, 8, 0, g10, 3) == 86
    # binomial barrier on 8 nodes: 3 (g + L) in, 3 (g + L) out
    assert plogp_sim.completion_time(17, 8, 8, 0, g10, 3) == 78


def test_exact_table_closed_forms():
    # g(z) = 32 + z / 8, L = 64: every intermediate is an integer (or a dyadic fraction)
    x = np.array([float(1 << i) for i in range(0, 21)])
    y = 32.0 + x / 8.0
    L = 64.0
    g1 = F(32) + F(1, 8)
    for m in (8, 64, 8000, 1 << 20, 3 << 22):
        for P in (2, 3, 4, 5, 8, 9, 64, 65, 66, 129, 1000, 4097):
            q, fl, cl = P - 1, flog2(P), clog2(P)
            want = {
                13: q * (32 + F(m, 8)) + F(L),
                14: 32 * q + F(m * P * (P - 1), 16) + q * F(L),
                15: 32 * cl + F(m * ((1 << cl) - 1), 8) + cl * F(L),
                16: 2 * (q * g1 + F(L)),
                17: 2 * (fl * g1 + cl * F(L)),
            }
            for sid, w in want.items():
                assert F(oracle.eval_strategy(x, y, L, sid, m, P)) == w, (sid, m, P)


def test_gather_rows_are_the_scatter_rows_bit_for_bit_and_barrier_ignores_m():
    rng = np.random.default_rng(5)
    for cfg in (1, 2, 5):
        wl = make_workload(cfg)
        x, y, L = wl.sizes[0], wl.gaps[0], float(wl.L[0])
        for _ in range(40):
            m = int(rng.choice(wl.m))
            P = int(rng.choice([2, 3, 5, 64, 65, 66, 200, 1000]))
            for a, b in ((10, 13), (11, 14), (12, 15)):
                assert bits(oracle.eval_strategy(x, y, L, a, m, P)) == bits(oracle.eval_strategy(x, y, L, b, m, P))
            for sid in (16, 17):
                assert bits(oracle.eval_strategy(x, y, L, sid, m, P)) == bits(oracle.eval_strategy(x, y, L, sid, 8, P))
        # every rounding of the Barrier rows made explicit
        g1 = rounded_g(x, y, 1)
        for P in (2, 3, 7, 8, 9, 1000):
            q, fl, cl = P - 1, flog2(P), clog2(P)
            assert oracle.eval_strategy(x, y, L, 16, 8, P) == rn(2 * F(rn(q * F(g1) + F(L))))
            assert oracle.eval_strategy(x, y, L, 17, 8, P) == rn(2 * F(rn(fl * F(g1) + F(rn(cl * F(L))))))


def test_planes_of_the_tuned_table_and_their_arg_min():
    wl = make_workload(2, m_slice=slice(3, 1024, 101), P_subset=[2, 3, 4, 7, 8, 9, 64, 65, 700])
    x, y, L = wl.sizes[0], wl.gaps[0], float(wl.L[0])
    full, _ = oracle.tune_grid(x, y, L, wl.m, wl.P, wl.s, wl.s_cap, 0x3FFFF)
    assert full.shape == (1, 4, len(wl.m), len(wl.P))
    base, _ = oracle.tune_grid(x, y, L, wl.m, wl.P, wl.s, wl.s_cap, 0x1FFF)
    assert full[:, :2].tobytes() == base.tobytes()               # the planes of Tables 1 and 2 are untouched
    # the Gather plane is the Scatter plane with its ids moved up by three
    assert (full["strategy"][0, 2] == full["strategy"][0, 1] + 3).all()
    assert bits(full["time"][0, 2]).tolist() == bits(full["time"][0, 1]).tolist()
    assert (full["s"][0, 2:] == 0).all()
    # brute force per cell over the plane's own rows, ties to the lowest id
    for op, ids in ((2, (13, 14, 15)), (3, (16, 17))):
        for mi, m in enumerate(wl.m):
            for pi, P in enumerate(wl.P):
                vals = [(oracle.eval_strategy(x, y, L, sid, int(m), int(P)), sid) for sid in ids]
                t, sid = min(vals)
                assert full["strategy"][0, op, mi, pi] == sid and full["time"][0, op, mi, pi] == t
    # two nodes: one hop in, one hop out either way: the Barrier rows tie and the flat one is named
    assert (full["strategy"][0, 3, :, 0] == 16).all()
    # the Barrier plane does not depend on the message size
    assert (full[0, 3] == full[0, 3, 0][None, :]).all()
    # a plane exists only if one of its rows is enabled; a subset of rows competes alone
    part, _ = oracle.tune_grid(x, y, L, wl.m, wl.P, wl.s, wl.s_cap, (1 << 14) | (1 << 15) | (1 << 17))
    assert part.shape[1] == 2
    assert set(np.unique(part["strategy"][0, 0])) <= {14, 15} and (part["strategy"][0, 1] == 17).all()
    ref, _ = oracle.tune_grid(x, y, L, wl.m, wl.P, wl.s, wl.s_cap, (1 << 11) | (1 << 12))
    assert bits(part["time"][0, 0]).tolist() == bits(ref["time"][0, 0]).tolist()
