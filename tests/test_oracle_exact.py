"""Pin P1: tables on which binary64 is exact, so each model value must equal an
integer/dyadic closed form derived by hand from Tables 1 and 2 -- independent
of any association order.  Also pins g() itself (index choice, clamping,
continuation above the last sample) against a plain count and exact
rationals."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from tests.helpers import F, clog2, exact_g, flog2, interval_linear, rounded_g


def affine_table(x0_exp=0, top_exp=24):
    x = np.array([float(1 << i) for i in range(x0_exp, top_exp + 1)])
    y = 32.0 + x / 8.0
    return x, y


L = 64.0


def closed_forms(m, P, s, g1):
    """Tables 1 and 2 for g(z) = 32 + z/8 in exact rationals."""
    g = lambda z: 32 + F(z) / 8
    q, fl, cl = P - 1, flog2(P), clog2(P)
    k = -(-m // s)
    R = 2 * F(g1) + 3 * F(L)
    return {
        0: q * g(m) + F(L),
        1: q * g(m) + R,
        2: q * (g(s) * k) + F(L),
        3: q * (g(m) + F(L)),
        4: q * (g(m) + R),
        5: q * (g(s) + F(L)) + g(s) * (k - 1),
        6: cl * (2 * g(m) + F(L)),
        7: fl * g(m) + cl * F(L),
        8: fl * g(m) + cl * R,
        9: fl * g(s) * k + cl * F(L),
        10: q * g(m) + F(L),
        # sum_{j=1}^{P-1} (32 + j m / 8) = 32 (P-1) + m P (P-1) / 16
        11: 32 * q + F(m * P * (P - 1), 16) + q * F(L),
        # sum_{j=0}^{cl-1} (32 + 2^j m / 8) = 32 cl + m (2^cl - 1) / 8
        12: 32 * cl + F(m * ((1 << cl) - 1), 8) + cl * F(L),
    }


@pytest.mark.parametrize("x0_exp", [0, 3])
def test_affine_table_every_row_is_exact(x0_exp):
    x, y = affine_table(x0_exp=x0_exp, top_exp=20)
    g1 = 32.125 if x0_exp == 0 else float(y[0])       # below the first sample: clamped
    for m in (8, 64, 1000 * 8, 1 << 20, 3 << 22, (1 << 30) + 8):
        for P in (2, 3, 4, 5, 7, 8, 9, 16, 17, 64, 65, 66, 129, 200, 1000):
            for s in (8, 24, 64, 4096, m):
                if s > m:
                    continue
                want = closed_forms(m, P, s, g1)
                for sid in range(13):
                    got = oracle.eval_strategy(x, y, L, sid, m, P, s)
                    assert F(got) == want[sid], (sid, m, P, s, got, float(want[sid]))


def test_scatter_chain_blocks_exact_beyond_many_blocks():
    # P - 1 = 64*b and 64*b +- 1 exercise the block boundaries
    x, y = affine_table(top_exp=16)
    for P in (64, 65, 66, 128, 129, 130, 4097, 65536):
        m = 1 << 10
        want = closed_forms(m, P, 8, 32.125)[11]
        got = oracle.eval_strategy(x, y, L, 11, m, P)
        assert F(got) == want


def test_tuned_scatter_rows_match_the_closed_forms_far_beyond_one_block():
    # the tuning forms the chain sums of all P in one pass over j (a prefix); with only the
    # chain row (or only the binomial row) enabled the table's times are that row's values:
    # they must equal the integer closed form and the one-point evaluation bit for bit,
    # at the block boundaries (P - 1 = 64 b and 64 b +- 1) up to 1023 blocks
    x, y = affine_table(top_exp=16)
    P = np.array([2, 3, 64, 65, 66, 128, 129, 130, 200, 4096, 4097, 4098, 65535, 65536], dtype=np.uint32)
    m = np.array([8, 1 << 10, 3 << 12], dtype=np.uint64)
    for sid in (11, 12):
        cells, _ = oracle.tune_grid(x, y, L, m, P, [], 0, 1 << sid)
        assert cells.shape == (1, 1, len(m), len(P))
        assert (cells["strategy"] == sid).all() and (cells["s"] == 0).all()
        for mi, mv in enumerate(m):
            for pi, Pv in enumerate(P):
                got = float(cells["time"][0, 0, mi, pi])
                assert F(got) == closed_forms(int(mv), int(Pv), 8, 32.125)[sid], (sid, mv, Pv)
                one = oracle.eval_strategy(x, y, L, sid, int(mv), int(Pv))
                assert np.float64(got).view(np.uint64) == np.float64(one).view(np.uint64)


def test_tuned_chain_sums_equal_the_one_point_sums_on_a_noisy_table():
    # the same on a table where the association order matters (sums are not exact): the
    # one-pass prefix of the tuning and the per-point sum must agree in every bit
    from plogp_workloads import make_workload
    wl = make_workload(5, m_slice=slice(7, 4096, 1361), P_subset=[2, 65, 66, 129, 4097, 40000, 65536])
    x, y, lat = wl.sizes[0], wl.gaps[0], float(wl.L[0])
    cells, _ = oracle.tune_grid(x, y, lat, wl.m, wl.P, [], 0, 1 << 11)
    for mi, mv in enumerate(wl.m):
        for pi, Pv in enumerate(wl.P):
            one = oracle.eval_strategy(x, y, lat, 11, int(mv), int(Pv))
            assert cells["time"][0, 0, mi, pi].view(np.uint64) == np.float64(one).view(np.uint64), (mv, Pv)


def test_g_hits_every_sample_and_matches_exact_rationals():
    # integer gaps y_i = i^2 on sizes 2^i: slopes (2i+1)/2^i are dyadic, so g is exact
    x = np.array([float(1 << i) for i in range(0, 21)])
    y = np.array([float(i * i) for i in range(0, 21)])
    for i, xi in enumerate(x):
        assert oracle.g(x, y, xi) == y[i]
    rng = np.random.default_rng(7)
    zs = list(rng.integers(1, 1 << 22, size=400)) + [1, 2, 3, (1 << 20) - 1, 1 << 20,
                                                     (1 << 20) + 1, 1 << 21, 5 << 20]
    for z in zs:
        z = int(z)
        assert F(oracle.g(x, y, z)) == exact_g(x, y, z), z


def test_g_at_a_sample_uses_the_interval_that_starts_there():
    # a sample belongs to the interval on its right, so g(x_i) = y_i with no
    # rounding at all; evaluated from the interval on its left it would come out
    # of slope * dx + y_{i-1}, which is off in the last bits when gaps cancel
    x = np.array([1.0, 4.0, 7.0, 11.0, 1024.0])
    y = np.array([1000.0, 0.001, 777.7, 1e-7, 3.3])
    for xi, yi in zip(x, y):
        assert oracle.g(x, y, xi) == yi
    left = [float(F(float((F(y[i]) - F(y[i - 1]))) / float(F(x[i]) - F(x[i - 1])))
                  * (F(x[i]) - F(x[i - 1])) + F(y[i - 1])) for i in range(1, 5)]
    assert any(l != yi for l, yi in zip(left, y[1:]))      # the case does discriminate


def test_g_index_is_last_sample_not_above_z():
    # irregular sizes: compare the interval the oracle must have used (via a
    # table whose gaps encode the interval index) with a plain count
    x = np.array([3.0, 4.0, 9.0, 10.0, 100.0, 101.0, 4096.0, 70000.0])
    y = np.array([0.0, 1000.0, 2000.0, 3000.0, 4000.0, 5000.0, 6000.0, 7000.0])
    for z in [1, 2, 3, 4, 5, 8, 9, 10, 11, 99, 100, 101, 102, 4095, 4096, 4097, 69999, 70000]:
        i = interval_linear(x, z)
        gz = oracle.g(x, y, z)
        lo = y[i]
        hi = y[min(i + 1, len(y) - 1)]
        assert lo <= gz <= hi if i < len(x) - 1 else gz >= lo
        if z in x:
            assert gz == y[list(x).index(z)]
    # below the first sample: clamped; above the last: the last line goes on
    assert oracle.g(x, y, 1) == 0.0
    slope_last = (7000.0 - 6000.0) / (70000.0 - 4096.0)
    assert oracle.g(x, y, 80000) == pytest.approx(7000.0 + slope_last * 10000.0, rel=1e-15)


def test_g_rounding_sequence_on_noisy_tables():
    from plogp_workloads import make_workload
    rng = np.random.default_rng(11)
    for cfg in (1, 2, 5):
        wl = make_workload(cfg)
        x, y = wl.sizes[0], wl.gaps[0]
        sl = oracle.slopes(x, y)
        for i in rng.integers(0, len(x) - 1, size=50):
            i = int(i)
            dy = float(F(y[i + 1]) - F(y[i])); dx = float(F(x[i + 1]) - F(x[i]))
            assert sl[i] == float(F(dy) / F(dx))
        assert sl[-1] == sl[-2]
        hi = int(x[-1]) * 4
        zs = [int(2.0 ** (np.log2(hi) * u)) + 1 for u in rng.random(300)]
        zs += [int(v) for v in x[:: max(1, len(x) // 40)]]
        for z in zs:
            assert oracle.g(x, y, z) == rounded_g(x, y, z), (cfg, z)
