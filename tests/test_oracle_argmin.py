"""Pins P3-P8 for the oracle's search: structural exact ties and the
tie-break, rational replay of every rounding, brute force on tiny grids, the
convex optimum of the segmented chain on an affine gap, the paper's
qualitative outcomes on a 100 Mbit/s-like table, metamorphic scalings."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from plogp_workloads import ALL_STRATEGIES_MASK, NO_CAP, SEGMENTED_IDS, make_workload
from tests.helpers import F, bits, exact_model_sum_forms, rounded_model


def noisy_table(cfg=2):
    wl = make_workload(cfg)
    return wl.sizes[0], wl.gaps[0], float(wl.L[0])


# ------------------------------------------------------------------ P3: ties

def test_two_nodes_make_flat_chain_binomial_tie_bitwise():
    x, y, L = noisy_table()
    for m in (8, 1024, 123456 * 8, 1 << 27):
        t = [oracle.eval_strategy(x, y, L, sid, m, 2) for sid in (0, 3, 7)]
        assert bits(t[0]) == bits(t[1]) == bits(t[2])
        t = [oracle.eval_strategy(x, y, L, sid, m, 2) for sid in (10, 11, 12)]
        assert bits(t[0]) == bits(t[1]) == bits(t[2])


def test_one_segment_ties_with_the_unsegmented_twin_and_scatter_flat_is_bcast_flat():
    x, y, L = noisy_table()
    for m in (8, 4096, 3 << 15):
        for P in (2, 3, 10, 64, 1000):
            for seg, plain in ((2, 0), (5, 3), (9, 7)):
                a = oracle.eval_strategy(x, y, L, seg, m, P, m)
                b = oracle.eval_strategy(x, y, L, plain, m, P)
                assert bits(a) == bits(b)
            assert bits(oracle.eval_strategy(x, y, L, 10, m, P)) == \
                bits(oracle.eval_strategy(x, y, L, 0, m, P))


def test_tie_break_lowest_id_then_unsegmented():
    x, y, L = noisy_table()
    m = np.array([4096, 65536], dtype=np.uint64)
    # P = 2: ids 0, 3, 7 tie; the table must name id 0 with s = 0
    out, _ = oracle.tune_grid(x, y, L, m, [2], [4096, 65536], NO_CAP, (1 << 0) | (1 << 3) | (1 << 7))
    assert (out["strategy"] == 0).all() and (out["s"] == 0).all()
    # only the segmented twins enabled with s = m as the single candidate: id 2 (lowest)
    out, _ = oracle.tune_grid(x, y, L, m[:1], [2], [4096], NO_CAP, (1 << 2) | (1 << 5) | (1 << 9))
    assert out["strategy"].item() == 2 and out["s"].item() == 4096
    # twin against its unsegmented row: the unsegmented (lower id) wins the tie
    out, _ = oracle.tune_grid(x, y, L, m[:1], [7], [4096], NO_CAP, (1 << 3) | (1 << 5))
    assert out["strategy"].item() == 3 and out["s"].item() == 0
    # equal times for two candidates (flat gap => g(s) k equal when s | m both times
    # only if gaps equal): a constant-gap table makes id 5 tie across no s, but id 2
    # gives g k, smallest at the largest s; check the smallest s wins among exact ties
    xc = np.array([1.0, 1 << 30]); yc = np.array([5.0, 5.0])
    out, _ = oracle.tune_grid(xc, yc, 0.0, [1 << 12], [5], [1 << 12, 1 << 13], NO_CAP, 1 << 2)
    assert out["s"].item() == 4096
    # duplicate candidates of equal cost: s = 2048 and 4096 with m = 2048*... not equal k;
    # a gap table with g(2s) = 2 g(s) exactly makes k g(s) tie for every s | m
    xl = np.array([1.0, 1 << 30]); yl = np.array([1.0, float(1 << 30)])
    out, _ = oracle.tune_grid(xl, yl, 3.0, [1 << 16], [9], [256, 1024, 4096, 1 << 16], NO_CAP, 1 << 2)
    assert out["strategy"].item() == 2 and out["s"].item() == 256


def test_no_enabled_strategy_and_no_valid_candidate():
    x, y, L = noisy_table()
    # segmented only, but every candidate is larger than m: nothing to choose
    out, _ = oracle.tune_grid(x, y, L, [64], [4], [128, 256], NO_CAP, 1 << 5)
    assert math.isinf(out["time"].item()) and out["strategy"].item() == 0xFFFFFFFF
    # candidate above the cap is skipped even if <= m
    out, _ = oracle.tune_grid(x, y, L, [4096], [4], [128, 1024], 512, 1 << 5)
    assert out["s"].item() == 128


# ------------------------------------------------------- P4: rational replay

@pytest.mark.parametrize("cfg", [1, 2, 4, 5])
def test_every_rounding_matches_rational_replay(cfg):
    wl = make_workload(cfg, n_tables=3) if cfg == 4 else make_workload(cfg)
    rng = np.random.default_rng(100 + cfg)
    x, y, L = wl.sizes[-1], wl.gaps[-1], float(wl.L[-1])
    Pmax_for_chain = 300
    for _ in range(60):
        m = int(rng.choice(wl.m)); P = int(rng.choice(wl.P))
        valid = [int(v) for v in wl.s if v <= min(m, wl.s_cap)]
        s = int(rng.choice(valid)) if valid else 0
        for sid in range(13):
            if sid in SEGMENTED_IDS and not valid:
                continue
            if sid == 11 and P > Pmax_for_chain:
                continue
            got = oracle.eval_strategy(x, y, L, sid, m, P, s)
            assert bits(got) == bits(rounded_model(x, y, L, sid, m, P, s)), (cfg, sid, m, P, s)


def test_scatter_sums_close_to_exact_rational_sums():
    # the blocked association order is a convention; whatever the order, the
    # value must be the mathematical sum to within a few units of roundoff
    wl = make_workload(5)
    x, y, L = wl.sizes[0], wl.gaps[0], float(wl.L[0])
    for m, P in ((8, 700), (4096, 2049), (1 << 20, 130), (40 * 8, 4097)):
        want = exact_model_sum_forms(x, y, L, 11, m, P)
        got = F(oracle.eval_strategy(x, y, L, 11, m, P))
        assert abs(got - want) <= Fraction(1, 10**13) * want
        want = exact_model_sum_forms(x, y, L, 12, m, P)
        got = F(oracle.eval_strategy(x, y, L, 12, m, P))
        assert abs(got - want) <= Fraction(1, 10**14) * want


# ---------------------------------------------------------- P5: brute force

@pytest.mark.parametrize("cfg", [1, 2, 5])
def test_tune_grid_equals_sorted_enumeration(cfg):
    wl = make_workload(cfg)
    rng = np.random.default_rng(cfg)
    m = np.sort(rng.choice(wl.m, size=6, replace=False))
    P = np.sort(rng.choice(wl.P[wl.P <= 200], size=5, replace=False)).astype(np.uint32)
    x, y, L = wl.sizes[0], wl.gaps[0], float(wl.L[0])
    out, _ = oracle.tune_grid(x, y, L, m, P, wl.s, wl.s_cap, wl.strategy_mask)
    ops = []
    if wl.strategy_mask & 0x3FF:
        ops.append(range(0, 10))
    if wl.strategy_mask & 0x1C00:
        ops.append(range(10, 13))
    for oi, ids in enumerate(ops):
        for mi, mv in enumerate(m):
            for pi, Pv in enumerate(P):
                cands = []
                for sid in ids:
                    if not (wl.strategy_mask >> sid) & 1:
                        continue
                    if sid in SEGMENTED_IDS:
                        for sv in wl.s:
                            if sv <= min(int(mv), wl.s_cap):
                                cands.append((oracle.eval_strategy(x, y, L, sid, int(mv), int(Pv), int(sv)),
                                              sid, int(sv)))
                    else:
                        cands.append((oracle.eval_strategy(x, y, L, sid, int(mv), int(Pv)), sid, 0))
                T, sid, sv = min(cands)
                c = out[0, oi, mi, pi]
                assert (bits(c["time"]), int(c["strategy"]), int(c["s"])) == (bits(T), sid, sv)


def test_duplicate_message_sizes_give_identical_rows():
    wl = make_workload(1)
    out, _ = oracle.tune_workload(wl)
    m = wl.m
    for i in range(1, len(m)):
        if m[i] == m[i - 1]:
            assert (out[0, 0, i].tobytes() == out[0, 0, i - 1].tobytes())


# ------------------------------------------- P6: convex optimum, affine gap

def test_segmented_chain_optimum_brackets_the_closed_form():
    # g(z) = g0 + z / Bw (dyadic so the table is exact); s | m.  Then
    # T5(s) = (P-2)(g0 + s/Bw) + (P-1) L + g0 m/s + m/Bw, convex in s with
    # minimum at s* = sqrt(g0 m Bw / (P-2)).
    g0, Bw, L = 32.0, 8.0, 64.0
    x = np.array([float(1 << i) for i in range(0, 31)])
    y = g0 + x / Bw
    m = 1 << 24
    cands = np.array([1 << j for j in range(3, 25)], dtype=np.uint64)
    for P in (3, 4, 10, 50, 1000):
        out, _ = oracle.tune_grid(x, y, L, [m], [P], cands, NO_CAP, 1 << 5)
        s_star = math.sqrt(g0 * m * Bw / (P - 2))
        lo = max(c for c in cands if c <= s_star)
        hi = min(c for c in cands if c >= s_star)
        assert out["s"].item() in (lo, hi), (P, s_star, out["s"].item())
    # two nodes: no pipeline to fill, T5 decreases with s, the best candidate is s = m
    out, _ = oracle.tune_grid(x, y, L, [m], [2], cands, NO_CAP, 1 << 5)
    assert out["s"].item() == m
    # ... and against its unsegmented twin the tie goes to the chain (id 3)
    out, _ = oracle.tune_grid(x, y, L, [m], [2], cands, NO_CAP, (1 << 3) | (1 << 5))
    assert out["strategy"].item() == 3


def test_segmented_flat_and_binomial_never_beat_their_twins_on_affine_gap():
    # with g0 >= 0, g(s) ceil(m/s) >= g(m): rows 2 and 9 cannot win
    x = np.array([float(1 << i) for i in range(0, 31)])
    y = 40.0 + x / 11.5
    m = np.array([8 * v for v in (1, 7, 100, 5000, 70000, 1 << 20)], dtype=np.uint64)
    P = np.array([2, 3, 9, 64, 500], dtype=np.uint32)
    s = np.array([8 << j for j in range(0, 20)], dtype=np.uint64)
    out, _ = oracle.tune_grid(x, y, 55.0, m, P, s, NO_CAP, ALL_STRATEGIES_MASK)
    assert not np.isin(out[0, 0]["strategy"], (2, 9)).any()


# -------------------------------------------- P7: the paper's own outcomes

def test_paper_outcomes_on_a_fast_ethernet_like_table():
    wl = make_workload(1)
    out, _ = oracle.tune_workload(wl)
    bc = out[0, 0]
    # Section 4.1: the segmented chain is the best Broadcast for large messages
    big = wl.m >= (256 << 10)
    manyP = wl.P >= 4
    assert (bc["strategy"][np.ix_(big, manyP)] == 5).all()
    # its segment size is a few kB, the order of the 8 kB of Fig. 1(b)
    s_big = bc["s"][np.ix_(wl.m == wl.m.max(), (wl.P >= 10))]
    assert s_big.min() >= 2048 and s_big.max() <= 16384
    # small messages go unsegmented
    assert (bc["s"][wl.m <= 256] == 0).all()
    # Section 4.2 on a noise-free copy, P a power of two: Binomial Scatter beats
    # Flat iff (P-1-log2 P) g0 > (log2 P - 1) L: loses at P = 4, wins at 8, 16, 32
    x = wl.sizes[0]
    y = 40.0 + x / 11.5
    P = np.array([4, 8, 16, 32], dtype=np.uint32)
    out, _ = oracle.tune_grid(x, y, 55.0, wl.m, P, wl.s, NO_CAP, (1 << 10) | (1 << 12))
    assert (out[0, 0]["strategy"][:, 0] == 10).all()
    assert (out[0, 0]["strategy"][:, 1:] == 12).all()


# ------------------------------------------------------- P8: metamorphic

def test_scaling_gaps_and_latency_by_a_power_of_two_scales_times_only():
    wl = make_workload(2, m_slice=slice(0, 1024, 37), P_subset=[2, 3, 17, 64, 100, 1024])
    a, _ = oracle.tune_workload(wl)
    b, _ = oracle.tune_grid(wl.sizes, wl.gaps * 8.0, wl.L * 8.0, wl.m, wl.P, wl.s, wl.s_cap,
                            wl.strategy_mask)
    assert (b["strategy"] == a["strategy"]).all() and (b["s"] == a["s"]).all()
    assert (bits(b["time"]) == bits(a["time"] * 8.0)).all()


def test_scaling_all_sizes_by_two_changes_nothing_but_s():
    wl = make_workload(2, m_slice=slice(0, 1024, 41), P_subset=[2, 5, 33, 257, 1000])
    a, _ = oracle.tune_workload(wl)
    b, _ = oracle.tune_grid(wl.sizes * 2.0, wl.gaps, wl.L, wl.m * np.uint64(2), wl.P,
                            wl.s * np.uint64(2), wl.s_cap * 2, wl.strategy_mask)
    # g(1) is the one size that does not scale with the table: on a table that
    # starts above 2 bytes it is clamped both times, so the rendezvous rows agree too
    assert wl.sizes[0, 0] >= 2
    assert (bits(b["time"]) == bits(a["time"])).all()
    assert (b["strategy"] == a["strategy"]).all() and (b["s"] == 2 * a["s"]).all()


def test_times_do_not_decrease_with_P_and_rendezvous_costs_more():
    x, y, L = noisy_table()
    for sid in range(13):
        for m, s in ((4096, 512), (1 << 22, 1 << 14)):
            prev = -1.0
            for P in range(2, 200):
                T = oracle.eval_strategy(x, y, L, sid, m, P, s)
                assert T >= prev, (sid, m, P)
                prev = T
    for plain, rdv in ((0, 1), (3, 4), (7, 8)):
        for P in (2, 9, 100):
            assert oracle.eval_strategy(x, y, L, rdv, 4096, P) > oracle.eval_strategy(x, y, L, plain, 4096, P)
