"""CPU oracle for the pLogP tuning sweep -- TEST INFRASTRUCTURE ONLY.

`plogp_oracle.c` is the plain implementation of what the hot path computes;
this module compiles it with gcc and exposes it through ctypes.  Only tests,
the smoke check and the benchmark's cpu_baseline leg may import it; the HIP
library never does and shares no code with it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "plogp_oracle.c"
_LIB = _HERE / "libplogp_oracle.so"

CELL_DTYPE = np.dtype([("time", "<f8"), ("s", "<u4"), ("strategy", "<u4")])
VERDICT_DTYPE = np.dtype([("regret", "<f8"), ("pred_best", "<u4"), ("meas_best", "<u4")])
SCORE_DTYPE = np.dtype([("sum_abs_err", "<f8"), ("max_abs_err", "<f8"), ("count", "<u8"),
                        ("reserved", "<u8")])

# strategy ids of each operation, in the order of the decision table's planes:
# Broadcast (Table 1), Scatter (Table 2), Gather, Barrier
OP_MASKS = (0x3FF, 0x1C00, 0xE000, 0x30000)

_lib = None


def build(force: bool = False) -> Path:
    """Compile the oracle (gcc, contraction off, fma only where written)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        cmd = ["gcc", "-std=c11", "-O2", "-mfma", "-ffp-contract=off", "-fno-fast-math",
               "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
               "-o", str(tmp), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        dp = ctypes.POINTER(ctypes.c_double)
        lib.plogp_oracle_slopes.argtypes = [dp, dp, ctypes.c_size_t, dp]
        lib.plogp_oracle_slopes.restype = None
        lib.plogp_oracle_g.argtypes = [dp, dp, ctypes.c_size_t, ctypes.c_double]
        lib.plogp_oracle_g.restype = ctypes.c_double
        lib.plogp_oracle_eval.argtypes = [dp, dp, ctypes.c_size_t, ctypes.c_double, ctypes.c_int,
                                          ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64, dp]
        lib.plogp_oracle_eval.restype = ctypes.c_int
        lib.plogp_oracle_tune.argtypes = [
            dp, dp, ctypes.c_size_t, dp, ctypes.c_size_t,
            ctypes.POINTER(ctypes.c_uint64), ctypes.c_size_t,
            ctypes.POINTER(ctypes.c_uint32), ctypes.c_size_t,
            ctypes.POINTER(ctypes.c_uint64), ctypes.c_size_t,
            ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_int]
        lib.plogp_oracle_tune.restype = ctypes.c_int
        lib.plogp_oracle_score.argtypes = [
            dp, dp, ctypes.c_size_t, ctypes.c_double,
            ctypes.POINTER(ctypes.c_uint64), ctypes.c_size_t,
            ctypes.POINTER(ctypes.c_uint32), ctypes.c_size_t, ctypes.c_uint32,
            dp, ctypes.POINTER(ctypes.c_uint32), dp, ctypes.c_void_p, ctypes.c_void_p]
        lib.plogp_oracle_score.restype = ctypes.c_int
        _lib = lib
    return _lib


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def slopes(x, y) -> np.ndarray:
    x = _f64(x); y = _f64(y)
    out = np.empty_like(x)
    _load().plogp_oracle_slopes(_dptr(x), _dptr(y), x.size, _dptr(out))
    return out


def g(x, y, z) -> float:
    """Gap at size z (piecewise-linear reading of the measured table)."""
    x = _f64(x); y = _f64(y)
    return float(_load().plogp_oracle_g(_dptr(x), _dptr(y), x.size, float(z)))


def eval_strategy(x, y, L, strategy: int, m: int, P: int, s: int = 0) -> float:
    """One model value (Table 1 / Table 2 row `strategy`)."""
    x = _f64(x); y = _f64(y)
    out = ctypes.c_double()
    rc = _load().plogp_oracle_eval(_dptr(x), _dptr(y), x.size, float(L), int(strategy),
                                   int(m), int(P), int(s), ctypes.byref(out))
    if rc != 0:
        raise ValueError("argument outside the model's domain")
    return out.value


def tune_grid(sizes, gaps, L, m, P, s, s_cap: int, strategy_mask: int, n_threads: int = 0):
    """Decision tables [n_tables, n_ops, n_m, n_P] (structured array) and the
    number of threads the run used."""
    sizes = np.atleast_2d(_f64(sizes)); gaps = np.atleast_2d(_f64(gaps))
    L = np.atleast_1d(_f64(L))
    m = np.ascontiguousarray(m, dtype=np.uint64)
    P = np.ascontiguousarray(P, dtype=np.uint32)
    s = np.ascontiguousarray(s, dtype=np.uint64)
    nt, n = sizes.shape
    n_ops = sum(1 for op_mask in OP_MASKS if strategy_mask & op_mask)
    out = np.zeros((nt, n_ops, m.size, P.size), dtype=CELL_DTYPE)
    used = _load().plogp_oracle_tune(
        _dptr(sizes), _dptr(gaps), n, _dptr(L), nt,
        m.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)), m.size,
        P.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), P.size,
        s.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)), s.size,
        ctypes.c_uint64(int(s_cap)), ctypes.c_uint32(int(strategy_mask)),
        out.ctypes.data_as(ctypes.c_void_p), int(n_threads))
    if used < 0:
        raise ValueError("bad argument to the oracle")
    return out, used


def tune_workload(wl, n_threads: int = 0):
    return tune_grid(wl.sizes, wl.gaps, wl.L, wl.m, wl.P, wl.s, wl.s_cap,
                     wl.strategy_mask, n_threads)


def strategy_ids(strategy_mask: int):
    """The enabled strategy ids, ascending (the row order of measurements and predictions)."""
    return [i for i in range(13) if (strategy_mask >> i) & 1]     # the measured rows: Tables 1 and 2


def score_grid(x, y, L, m, P, strategy_mask: int, meas, seg):
    """Prediction against measurement (see plogp_oracle_score): returns
    (pred [n_ids, n_m, n_P], verdict [n_ops, n_m, n_P], score [n_ids])."""
    x = _f64(x); y = _f64(y)
    m = np.ascontiguousarray(m, dtype=np.uint64)
    P = np.ascontiguousarray(P, dtype=np.uint32)
    n_ids = len(strategy_ids(strategy_mask))
    meas = np.ascontiguousarray(meas, dtype=np.float64)
    seg = np.ascontiguousarray(seg, dtype=np.uint32)
    assert meas.shape == (n_ids, m.size, P.size) and seg.shape == meas.shape
    n_ops = (1 if strategy_mask & 0x3FF else 0) + (1 if strategy_mask & 0x1C00 else 0)   # Tables 1 and 2 only
    pred = np.empty_like(meas)
    verdict = np.zeros((n_ops, m.size, P.size), dtype=VERDICT_DTYPE)
    score = np.zeros(n_ids, dtype=SCORE_DTYPE)
    rc = _load().plogp_oracle_score(
        _dptr(x), _dptr(y), x.size, float(L),
        m.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)), m.size,
        P.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), P.size, ctypes.c_uint32(int(strategy_mask)),
        _dptr(meas), seg.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), _dptr(pred),
        verdict.ctypes.data_as(ctypes.c_void_p), score.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError("bad argument to the oracle")
    return pred, verdict, score
