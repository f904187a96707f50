"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every function the headers under include/ declare, and refuses bad arguments before it
ever touches the device.  (With no GPU, a valid call must fail loudly with
PLOGP_EDEVICE: there is no CPU fallback.)"""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def plogp():
    from paper_cs_0408034_amd import build
    build.build_library(force=False)
    from paper_cs_0408034_amd import plogp as mod
    return mod


def declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(inc, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(plogp_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(plogp):
    names = declared_functions()
    assert {"plogp_load_table", "plogp_eval_strategy", "plogp_tune_grid", "plogp_tune_grid_profile",
            "plogp_measure_ceilings"} <= set(names)
    lib = ctypes.CDLL(str(plogp.LIB_PATH))
    for name in names:
        assert hasattr(lib, name), name


def test_cell_is_sixteen_bytes(plogp):
    assert plogp.CELL_DTYPE.itemsize == 16
    assert plogp.CELL_DTYPE.fields["s"][1] == 8 and plogp.CELL_DTYPE.fields["strategy"][1] == 12


def test_strerror_covers_every_status(plogp):
    msgs = {plogp._lib.plogp_strerror(i).decode() for i in range(7)}
    assert len(msgs) == 7 and "unknown status" not in msgs
    assert plogp._lib.plogp_strerror(99).decode() == "unknown status"


def _status(plogp, fn, *a, **k):
    try:
        fn(*a, **k)
    except plogp.PlogpError as e:
        return e.status
    return plogp.OK


GOOD_X = [1.0, 8.0, 64.0]
GOOD_Y = [1.0, 2.0, 3.0]


@pytest.mark.parametrize("x,y,L", [
    ([1.0, 8.0], [1.0, float("nan")], 1.0),            # NaN gap
    ([1.0, 8.0], [1.0, -2.0], 1.0),                    # negative gap
    ([1.0, 8.0], [1.0, float("inf")], 1.0),
    ([1.0, 8.0], [1.0, 2.0 ** 801], 1.0),              # a gap so large that a model could overflow
    (GOOD_X, GOOD_Y, 2.0 ** 801),
    ([1.0, 1.0], [1.0, 2.0], 1.0),                     # sizes not strictly increasing
    ([8.0, 1.0], [1.0, 2.0], 1.0),
    ([0.0, 8.0], [1.0, 2.0], 1.0),                     # size below one byte
    ([1.5, 8.0], [1.0, 2.0], 1.0),                     # not an integer
    ([1.0, 2.0 ** 53], [1.0, 2.0], 1.0),               # not exact in binary64
    ([1.0], [1.0], 1.0),                               # fewer than two samples
    (GOOD_X, GOOD_Y, -1.0), (GOOD_X, GOOD_Y, float("nan")),
])
def test_load_table_rejects(plogp, x, y, L):
    assert _status(plogp, plogp.plogp_load_table, x, y, L) == plogp.EINVAL


def test_load_table_rejects_too_many_samples_and_null(plogp):
    x = np.arange(1, plogp.MAX_SAMPLES + 2, dtype=np.float64)
    assert _status(plogp, plogp.plogp_load_table, x, x, 1.0) == plogp.EINVAL
    h = ctypes.c_void_p()
    assert plogp._lib.plogp_load_table(None, None, 3, 1.0, ctypes.byref(h)) == plogp.EINVAL
    assert plogp._lib.plogp_load_tables(None, None, 3, None, 1, ctypes.byref(h)) == plogp.EINVAL
    assert h.value is None


@pytest.mark.parametrize("kw", [
    dict(m=[0], P=[2], s=[8]),                         # m = 0
    dict(m=[8], P=[1], s=[8]),                         # P < 2
    dict(m=[8], P=[4, 4], s=[8]),                      # P not strictly ascending
    dict(m=[8], P=[4, 3], s=[8]),
    dict(m=[8], P=[2], s=[0]),                         # s = 0
    dict(m=[8], P=[2], s=[16, 8]),                     # candidates not ascending
    dict(m=[8], P=[2], s=[8, 8]),
    dict(m=[12], P=[2], s=[8]),                        # m not a multiple of the datatype
    dict(m=[16], P=[2], s=[4]),                        # s not a multiple of the datatype
    dict(m=[8], P=[2], s=[1 << 32]),                   # s does not fit the record
    dict(m=[8], P=[2], s=[8], strategy_mask=0),        # nothing to evaluate
    dict(m=[8], P=[2], s=[8], strategy_mask=1 << 18),  # unknown strategy
    dict(m=[], P=[2], s=[8]), dict(m=[8], P=[], s=[8]),
])
def test_grid_create_rejects(plogp, kw):
    assert _status(plogp, plogp.plogp_grid_create, **kw) == plogp.EINVAL


def test_grid_create_range_errors(plogp):
    assert _status(plogp, plogp.plogp_grid_create, m=[1 << 53], P=[2], s=[8]) == plogp.ERANGE
    # chain scatter: (Pmax - 1) * m would reach 2^53
    assert _status(plogp, plogp.plogp_grid_create, m=[1 << 40], P=[2, 1 << 14], s=[8]) == plogp.ERANGE
    # the same grid without the Scatter rows is fine as far as validation goes
    st = _status(plogp, plogp.plogp_grid_create, m=[1 << 40], P=[2, 1 << 14], s=[8],
                 strategy_mask=plogp.MASK_BCAST)
    assert st in (plogp.OK, plogp.EDEVICE)
    # binomial scatter alone: 2^(ceil(log2 Pmax) - 1) * m
    assert _status(plogp, plogp.plogp_grid_create, m=[1 << 40], P=[1 << 14], s=[8],
                   strategy_mask=1 << 12) == plogp.ERANGE
    # the Gather twins of those rows add up the same sizes
    for sid in (14, 15):
        assert _status(plogp, plogp.plogp_grid_create, m=[1 << 40], P=[2, 1 << 14], s=[8],
                       strategy_mask=1 << sid) == plogp.ERANGE
    # a Barrier carries no payload: any size below 2^53 goes
    st = _status(plogp, plogp.plogp_grid_create, m=[1 << 40], P=[2, 1 << 14], s=[8],
                 strategy_mask=plogp.MASK_BARRIER)
    assert st in (plogp.OK, plogp.EDEVICE)


def test_null_handles_are_refused(plogp):
    lib = plogp._lib
    assert lib.plogp_tune_grid(None, None, None, 0, None) == plogp.EINVAL
    assert lib.plogp_interp_g(None, 0, None, 1, None, None) == plogp.EINVAL
    assert lib.plogp_eval_strategy(None, 0, 0, None, None, None, 1, None, None) == plogp.EINVAL
    assert lib.plogp_grid_create(None, None) == plogp.EINVAL
    assert lib.plogp_table_count(None) == 0 and lib.plogp_decision_table_bytes(3, None) == 0
    assert lib.plogp_free_table(None) == plogp.OK and lib.plogp_grid_free(None) == plogp.OK
    assert lib.plogp_cutovers(None, 1, None, 0, None, None, 0, None) == plogp.EINVAL
    assert lib.plogp_cutovers_profile(None, 1, None, 0, None, None, 0, None, 1, None) == plogp.EINVAL
    assert lib.plogp_cutover_rows(3, None) == 0
    assert lib.plogp_score_grid(None, 0, None, None, None, None, None, None, None) == plogp.EINVAL
    assert lib.plogp_score_grid_profile(None, 0, None, None, None, None, None, None, None, 1, None) == plogp.EINVAL
    assert lib.plogp_score_strategies(None) == 0
    assert lib.plogp_robustness(None, 1, None, 0, None, None, None, None) == plogp.EINVAL
    assert lib.plogp_robustness_profile(None, 1, None, 0, None, None, None, None, 1, None) == plogp.EINVAL


def test_verdict_and_score_records(plogp):
    assert plogp.VERDICT_DTYPE.itemsize == 16 and plogp.SCORE_DTYPE.itemsize == 32


def test_run_is_sixteen_bytes(plogp):
    assert plogp.RUN_DTYPE.itemsize == 16
    assert plogp.RUN_DTYPE.fields["s"][1] == 8 and plogp.RUN_DTYPE.fields["strategy"][1] == 12


def test_without_a_gpu_valid_calls_fail_loudly(plogp):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    assert _status(plogp, plogp.plogp_load_table, GOOD_X, GOOD_Y, 1.0) == plogp.EDEVICE
    assert plogp._lib.plogp_last_hip_error() != 0
    assert _status(plogp, plogp.plogp_grid_create, m=[8], P=[2], s=[8]) == plogp.EDEVICE
