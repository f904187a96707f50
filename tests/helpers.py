"""Exact-arithmetic helpers shared by the CPU tests (no code of the oracle or
of the HIP library is used here)."""
from __future__ import annotations

from fractions import Fraction

import numpy as np


def F(v, d=1) -> Fraction:
    return Fraction(v) / Fraction(d)


def rn(v: Fraction) -> float:
    """Round an exact value to binary64, ties to even (float(Fraction) is exact)."""
    return float(v)


def flog2(P: int) -> int:
    return P.bit_length() - 1


def clog2(P: int) -> int:
    return (P - 1).bit_length()


def interval_linear(x, z) -> int:
    """Index of the last sample <= z by a plain count, clamped to [0, n-1]."""
    cnt = sum(1 for xi in x if xi <= z)
    return max(cnt - 1, 0)


def exact_g(x, y, z) -> Fraction:
    """Piecewise-linear gap in exact rational arithmetic (exact slopes):
    clamped below the first sample, last line continued above the last."""
    n = len(x)
    i = interval_linear(x, z)
    seg = min(i, n - 2)
    slope = (F(y[seg + 1]) - F(y[seg])) / (F(x[seg + 1]) - F(x[seg]))
    zc = max(F(z), F(x[0]))
    return F(y[i]) + slope * (zc - F(x[i]))


def rounded_g(x, y, z) -> float:
    """The gap with every rounding of the binary64 evaluation made explicit:
    slope = rn(rn(dy) / rn(dx)); g = rn(slope * (zc - x_i) + y_i) (one fma)."""
    n = len(x)
    i = interval_linear(x, z)
    seg = min(i, n - 2)
    dy = rn(F(y[seg + 1]) - F(y[seg]))
    dx = rn(F(x[seg + 1]) - F(x[seg]))
    slope = rn(F(dy) / F(dx))
    zc = max(float(z), float(x[0]))
    d = rn(F(zc) - F(x[i]))
    return rn(F(slope) * F(d) + F(y[i]))


def rounded_model(x, y, L, sid, m, P, s=0) -> float:
    """Tables 1 and 2 with each multiplication, addition and fused
    multiply-add rounded once, computed in rational arithmetic."""
    g = lambda z: rounded_g(x, y, z)
    q, fl, cl = P - 1, flog2(P), clog2(P)
    gm, g1 = g(m), g(1)
    R = rn(3 * F(L) + F(rn(2 * F(g1))))
    if sid in (2, 5, 9):
        gs = g(s)
        k = -(-m // s)
        A = rn(F(gs) * k)
        B = rn(F(gs) * (k - 1))
        C = rn(F(gs) + F(L))
    if sid in (0, 10):
        return rn(q * F(gm) + F(L))
    if sid == 1:
        return rn(q * F(gm) + F(R))
    if sid == 2:
        return rn(q * F(A) + F(L))
    if sid == 3:
        return rn(q * F(rn(F(gm) + F(L))))
    if sid == 4:
        return rn(q * F(rn(F(gm) + F(R))))
    if sid == 5:
        return rn(q * F(C) + F(B))
    if sid == 6:
        return rn(cl * F(rn(2 * F(gm) + F(L))))
    if sid == 7:
        return rn(fl * F(gm) + F(rn(cl * F(L))))
    if sid == 8:
        return rn(fl * F(gm) + F(rn(cl * F(R))))
    if sid == 9:
        return rn(fl * F(A) + F(rn(cl * F(L))))
    if sid == 11:
        done, run = 0.0, 0.0
        for j in range(1, P):
            run = rn(F(run) + F(g(j * m)))
            if j % 64 == 0:
                done = rn(F(done) + F(run))
                run = 0.0
        S = rn(F(done) + F(run))
        return rn(q * F(L) + F(S))
    if sid == 12:
        S = 0.0
        for j in range(cl):
            S = rn(F(S) + F(g(m << j)))
        return rn(cl * F(L) + F(S))
    raise ValueError(sid)


def exact_model_sum_forms(x, y, L, sid, m, P) -> Fraction:
    """Scatter rows with exact g and exact sums (no rounding anywhere)."""
    if sid == 11:
        return sum(exact_g(x, y, j * m) for j in range(1, P)) + (P - 1) * F(L)
    if sid == 12:
        cl = clog2(P)
        return sum(exact_g(x, y, m << j) for j in range(cl)) + cl * F(L)
    raise ValueError(sid)


def bits(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64).view(np.uint64)
