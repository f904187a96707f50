"""The seeded generator is deterministic and has the shapes the five configs
state; the oracle still reproduces the stored config-1 values."""
import os

import numpy as np
import pytest

import oracle
from plogp_workloads import SplitMix64, make_workload

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_splitmix64_reference_values():
    # first outputs of splitmix64 seeded with 0 and with 1234567 (published test vectors)
    r = SplitMix64(0)
    assert [r.next_u64() for _ in range(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4,
                                                0x06C45D188009454F]
    r = SplitMix64(1234567)
    assert [r.next_u64() for _ in range(2)] == [6457827717110365317, 3203168211198807973]
    a = SplitMix64(99); b = SplitMix64(99)
    assert [a.uniform() for _ in range(10)] == list(b.uniforms(10))
    assert a.state == b.state


@pytest.mark.parametrize("cfg,shape", [
    (1, (1, 21, 64, 49, 13)), (2, (1, 64, 1024, 1023, 34)), (3, (1, 64, 1024, 69, 8192)),
    (5, (1, 4096, 4096, 712, 42))])
def test_shapes(cfg, shape):
    wl = make_workload(cfg)
    assert (wl.n_tables, wl.sizes.shape[1], len(wl.m), len(wl.P), len(wl.s)) == shape
    assert (np.diff(wl.sizes[0]) > 0).all() and (np.diff(wl.gaps[0]) >= 0).all()
    assert (np.diff(wl.P.astype(np.int64)) > 0).all() and (np.diff(wl.s.astype(np.int64)) > 0).all()
    assert (wl.m % 8 == 0).all() and (wl.s % 8 == 0).all() and wl.m.min() >= 8


def test_counts_match_the_enumerated_grid_sizes():
    want = {1: (3136, 21805, 163072), 2: (2095104, 79813437, 463017984),
            3: (141312, 1737148416, 7524581376), 5: (5832704, 260035216, 1592328192)}
    for cfg, (cells, eff, nom) in want.items():
        c = make_workload(cfg).counts()
        assert (c["cells"], c["effective_evals"], c["nominal_evals"]) == (cells, eff, nom)
    c = make_workload(4, n_tables=10).counts()
    assert c["cells"] == 10 * 2 * 256 * 24 and c["effective_evals"] == 2299200
    assert c["scatter_chain_interps"] == 10 * 256 * 511


def test_config4_tables_are_seeded_per_table():
    a = make_workload(4, n_tables=5)
    b = make_workload(4, n_tables=2, table_offset=3)
    assert np.array_equal(a.gaps[3:], b.gaps) and np.array_equal(a.L[3:], b.L)
    assert 2.0 <= a.L.min() and a.L.max() <= 100.0


def test_stored_config1_values():
    wl = make_workload(1)
    with open(os.path.join(GOLD, "cfg1_table.txt")) as f:
        rows = [ln.split() for ln in f if not ln.startswith("#")]
    assert [int(r[0]) for r in rows] == [int(v) for v in wl.sizes[0]]
    assert [float.fromhex(r[1]) for r in rows] == list(wl.gaps[0])
    out, _ = oracle.tune_workload(wl)
    with open(os.path.join(GOLD, "cfg1_decisions.txt")) as f:
        rows = [ln.split() for ln in f if not ln.startswith("#")]
    assert len(rows) > 100
    for r in rows:
        mi, mb, P, sid, s = (int(v) for v in r[:5])
        c = out[0, 0, mi, int(P) - 2]
        assert int(wl.m[mi]) == mb
        assert (int(c["strategy"]), int(c["s"]), float(c["time"])) == (sid, s, float.fromhex(r[5]))


def test_measurement_and_perturbation_generators_are_seeded_and_model_free():
    """The synthetic measured times and the perturbed parameter sets: reproducible, of the
    stated shapes and ranges, and built without any of the method's arithmetic."""
    from plogp_workloads import make_measurements, make_perturbed
    wl = make_workload(1)
    meas, seg = make_measurements(wl, seed=4)
    meas2, seg2 = make_measurements(wl, seed=4)
    n_ids = bin(wl.strategy_mask).count("1")
    assert meas.shape == seg.shape == (n_ids, len(wl.m), len(wl.P))
    assert meas.dtype == np.float64 and seg.dtype == np.uint32
    assert (meas == meas2).all() and (seg == seg2).all()
    assert not (make_measurements(wl, seed=5)[0] == meas).all()
    assert (meas > 0).all() and np.isfinite(meas).all()
    m = wl.m.astype(np.uint64)[None, :, None]
    assert (seg >= 1).all() and (seg <= m).all() and (seg <= 8192).all()
    assert ((seg & (seg - 1)) == 0).all()                       # powers of two
    pw = make_perturbed(wl, 5, 0.1, seed=2)
    pw2 = make_perturbed(wl, 5, 0.1, seed=2)
    assert pw.n_tables == 6 and (pw.gaps == pw2.gaps).all() and (pw.L == pw2.L).all()
    assert (pw.sizes == wl.sizes[0]).all() and (pw.gaps[0] == wl.gaps[0]).all() and pw.L[0] == wl.L[0]
    ratio = pw.gaps[1:] / wl.gaps[0]
    assert ratio.min() >= 0.9 and ratio.max() <= 1.1 and len(np.unique(ratio)) > 50
    assert (pw.m == wl.m).all() and (pw.P == wl.P).all() and (pw.s == wl.s).all()
    # no model inside the generator: the measured times do not depend on the table at all
    other = make_workload(1)
    other.gaps = other.gaps * 3.0
    other.L = other.L * 0.5
    assert (make_measurements(other, seed=4)[0] == meas).all()
