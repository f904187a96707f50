"""The five synthetic tuning workloads, plus free-form variants for tests.

Generator conventions (fixed so that two runs produce the same bytes):
  * PRNG: splitmix64; U(0,1) = (next() >> 11) * 2**-53.
  * seed = 408034000000 + 1_000_000 * config + table_index.
  * draw order per table: [sample positions, if random] then [L, g0, Bw, if
    random] then the n noise draws u_0..u_{n-1} then [breakpoints, jumps].
  * gap samples: y_i = g0 + (x_i / Bw) * (1 + noise * u_i), then the jumps,
    then a running maximum so the table is non-decreasing.
  * "n log-spaced sizes from lo to hi": m_i = max(8, 8*floor(lo*(hi/lo)**(i/(n-1)) / 8)),
    duplicates kept (the grid shape is fixed).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

STRATEGY_NAMES = (
    "bcast_flat",              # 0
    "bcast_flat_rdv",          # 1
    "bcast_flat_seg",          # 2
    "bcast_chain",             # 3
    "bcast_chain_rdv",         # 4
    "bcast_chain_seg",         # 5
    "bcast_binary",            # 6
    "bcast_binomial",          # 7
    "bcast_binomial_rdv",      # 8
    "bcast_binomial_seg",      # 9
    "scatter_flat",            # 10
    "scatter_chain",           # 11
    "scatter_binomial",        # 12
)
BCAST_IDS = tuple(range(0, 10))
SCATTER_IDS = (10, 11, 12)
SEGMENTED_IDS = (2, 5, 9)
ALL_STRATEGIES_MASK = (1 << 13) - 1
NO_CAP = (1 << 64) - 1          # s_cap value meaning "only s <= m limits the candidates"

_MASK64 = (1 << 64) - 1


class SplitMix64:
    """splitmix64 stream (public-domain generator by S. Vigna)."""

    def __init__(self, seed: int):
        self.state = seed & _MASK64

    def next_u64(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & _MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
        return z ^ (z >> 31)

    def uniform(self) -> float:
        return (self.next_u64() >> 11) * (1.0 / 9007199254740992.0)

    def uniforms(self, n: int) -> np.ndarray:
        """n consecutive uniform() draws, vectorised (same values, same order)."""
        with np.errstate(over="ignore"):
            k = np.arange(1, n + 1, dtype=np.uint64)
            z = np.uint64(self.state) + k * np.uint64(0x9E3779B97F4A7C15)
            self.state = int(z[-1]) if n else self.state
            z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
            z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
            z = z ^ (z >> np.uint64(31))
        return (z >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


@dataclass
class Workload:
    """One tuning job: a batch of pLogP tables and one grid shared by all of them."""

    name: str
    sizes: np.ndarray            # float64 [n_tables, n]   sample sizes x (bytes, integers)
    gaps: np.ndarray             # float64 [n_tables, n]   gap samples y (microseconds)
    L: np.ndarray                # float64 [n_tables]      latency (microseconds)
    m: np.ndarray                # uint64  [n_m]           message sizes (bytes)
    P: np.ndarray                # uint32  [n_P]           process counts, strictly ascending
    s: np.ndarray                # uint64  [n_s]           segment candidates, strictly ascending
    s_cap: int                   # candidate valid iff s <= min(m, s_cap)
    strategy_mask: int           # bit i = strategy id i takes part
    dtype_size: int = 8
    notes: dict = field(default_factory=dict)

    @property
    def n_tables(self) -> int:
        return int(self.sizes.shape[0])

    @property
    def n_ops(self) -> int:
        # planes of the decision table: Broadcast (ids 0..9), Scatter (10..12), Gather (13..15),
        # Barrier (16, 17), each present if one of its ids is enabled
        return sum(1 for op_mask in (0x3FF, 0x1C00, 0xE000, 0x30000) if self.strategy_mask & op_mask)

    @property
    def n_cells(self) -> int:
        return self.n_tables * self.n_ops * len(self.m) * len(self.P)

    def counts(self) -> dict:
        """Evaluation counts used by the throughput metric.

        effective = closed forms actually needed: every enabled unsegmented row
        once per (m, P) and every enabled segmented row once per valid (m, P, s);
        nominal = |strategies| * |m| * |P| * |s|, the dense product.
        interps = terms of the Scatter-chain sum when shared per m (P_max - 1 each).
        """
        mask = self.strategy_mask
        n_unseg = sum(1 for i in range(18) if (mask >> i) & 1 and i not in SEGMENTED_IDS)
        n_seg = sum(1 for i in SEGMENTED_IDS if (mask >> i) & 1)
        lim = np.minimum(self.m, np.uint64(self.s_cap))
        valid = np.searchsorted(self.s, lim, side="right")          # valid candidates per m
        n_ms = int(valid.sum())
        nP = len(self.P)
        eff = self.n_tables * (len(self.m) * nP * n_unseg + n_ms * nP * n_seg)
        nom = self.n_tables * bin(mask).count("1") * len(self.m) * nP * len(self.s)
        interps = 0
        if (mask >> 11) & 1 or (mask >> 14) & 1:
            interps = self.n_tables * len(self.m) * (int(self.P.max()) - 1)
        return {
            "cells": self.n_cells,
            "effective_evals": int(eff),
            "nominal_evals": int(nom),
            "ms_pairs": self.n_tables * n_ms,
            "scatter_chain_interps": int(interps),
            "output_bytes": self.n_cells * 16,
        }


def log_spaced_sizes(n: int, lo: float, hi: float) -> np.ndarray:
    out = np.empty(n, dtype=np.uint64)
    ratio = hi / lo
    for i in range(n):
        v = lo * ratio ** (i / (n - 1)) if n > 1 else lo
        out[i] = max(8, 8 * int(v // 8))
    return out


def _gap_table(x: np.ndarray, g0: float, bw: float, noise: float, u: np.ndarray,
               jumps=None) -> np.ndarray:
    y = g0 + (x / bw) * (1.0 + noise * u)
    if jumps:
        for b, jmp in jumps:
            y = y + np.where(x >= b, jmp, 0.0)
    return np.maximum.accumulate(y)


def _d2_sizes() -> np.ndarray:
    # 64 samples round(2**(i/2.5)), i = 7..70: 7 B ... 2**28 B = 256 MiB
    return np.array([float(round(2.0 ** (i / 2.5))) for i in range(7, 71)], dtype=np.float64)


def _pow2_set(lo_exp: int, hi_exp: int) -> list:
    return [1 << j for j in range(lo_exp, hi_exp + 1)]


def _seed(cfg: int, table_index: int = 0) -> int:
    return 408034000000 + 1_000_000 * cfg + table_index


def make_workload(cfg: int, *, n_tables: Optional[int] = None, n_m: Optional[int] = None,
                  m_slice: Optional[slice] = None, P_subset: Optional[np.ndarray] = None,
                  s_subset: Optional[slice] = None, table_offset: int = 0) -> Workload:
    """Build config `cfg` (1..5).  The keyword arguments cut a smaller job out of
    the same recipe for tests: fewer tables (config 4), a slice of the m list, a
    subset of P or of the s candidates.  `n_m` re-spaces the m list with n_m
    points over the same range instead."""
    if cfg == 1:
        x = np.array([float(1 << i) for i in range(21)])
        rng = SplitMix64(_seed(1))
        u = rng.uniforms(21)
        y = _gap_table(x, 40.0, 11.5, 0.03, u)
        wl = Workload(
            name="cfg1",
            sizes=x[None, :], gaps=y[None, :], L=np.array([55.0]),
            m=log_spaced_sizes(n_m or 64, 1.0, float(1 << 20)),
            P=np.arange(2, 51, dtype=np.uint32),
            s=np.array(_pow2_set(8, 20), dtype=np.uint64),
            s_cap=NO_CAP,
            strategy_mask=(1 << 0) | (1 << 3) | (1 << 7) | (1 << 5),
        )
    elif cfg in (2, 3):
        x = _d2_sizes()
        rng = SplitMix64(_seed(2))           # config 3 reuses config 2's table
        u = rng.uniforms(64)
        y = _gap_table(x, 40.0, 11.5, 0.03, u)
        if cfg == 2:
            s = sorted(set(_pow2_set(3, 20)) | {3 << j for j in range(3, 19)})
            wl = Workload(
                name="cfg2",
                sizes=x[None, :], gaps=y[None, :], L=np.array([55.0]),
                m=log_spaced_sizes(n_m or 1024, 8.0, float(1 << 28)),
                P=np.arange(2, 1025, dtype=np.uint32),
                s=np.array(s, dtype=np.uint64),
                s_cap=1 << 20,
                strategy_mask=ALL_STRATEGIES_MASK,
            )
        else:
            P = list(range(2, 65)) + [1 << a for a in range(7, 13)]
            wl = Workload(
                name="cfg3",
                sizes=x[None, :], gaps=y[None, :], L=np.array([55.0]),
                m=log_spaced_sizes(n_m or 1024, float(1 << 16), float(1 << 30)),
                P=np.array(P, dtype=np.uint32),
                s=np.arange(8, 65536 + 1, 8, dtype=np.uint64),
                s_cap=1 << 16,
                strategy_mask=ALL_STRATEGIES_MASK,
            )
    elif cfg == 4:
        nt = n_tables or 10000
        x = _d2_sizes()
        xs = np.empty((nt, 64)); ys = np.empty((nt, 64)); Ls = np.empty(nt)
        for t in range(nt):
            rng = SplitMix64(_seed(4, table_offset + t))
            d = rng.uniforms(3 + 64)
            Ls[t] = 2.0 + 98.0 * d[0]
            g0 = 1.0 + 49.0 * d[1]
            bw = 100.0 * 250.0 ** d[2]
            xs[t] = x
            ys[t] = _gap_table(x, g0, bw, 0.03, d[3:])
        Pl = [2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65,
              127, 128, 129, 255, 256, 257, 511, 512]
        wl = Workload(
            name="cfg4",
            sizes=xs, gaps=ys, L=Ls,
            m=log_spaced_sizes(n_m or 256, 8.0, float(1 << 26)),
            P=np.array(Pl, dtype=np.uint32),
            s=np.array(_pow2_set(6, 26), dtype=np.uint64),
            s_cap=NO_CAP,
            strategy_mask=ALL_STRATEGIES_MASK,
        )
    elif cfg == 5:
        rng = SplitMix64(_seed(5))
        seen = {1, 1 << 32}
        while len(seen) < 4096:
            seen.add(int(2.0 ** (32.0 * rng.uniform())))
        x = np.array(sorted(seen), dtype=np.float64)
        u = rng.uniforms(4096)
        bps = [float(int(2.0 ** (10.0 + 16.0 * rng.uniform()))) for _ in range(4)]
        jps = [5.0 + 25.0 * rng.uniform() for _ in range(4)]
        y = _gap_table(x, 40.0, 11.5, 0.05, u, jumps=list(zip(bps, jps)))
        Pset = {1 << a for a in range(1, 17)}
        for a in range(1, 16):
            for t in range(1, 65):
                p = (1 << a) + int(round(t * (1 << a) / 65.0))
                if (1 << a) < p < (1 << (a + 1)):
                    Pset.add(p)
        s = sorted(set(_pow2_set(3, 24)) | {3 << j for j in range(3, 23)})
        wl = Workload(
            name="cfg5",
            sizes=x[None, :], gaps=y[None, :], L=np.array([55.0]),
            m=log_spaced_sizes(n_m or 4096, 8.0, float(1 << 32)),
            P=np.array(sorted(Pset), dtype=np.uint32),
            s=np.array(s, dtype=np.uint64),
            s_cap=1 << 24,
            strategy_mask=ALL_STRATEGIES_MASK,
            notes={"breakpoints": bps, "jumps": jps},
        )
    else:
        raise ValueError("config must be 1..5")

    if m_slice is not None:
        wl.m = np.ascontiguousarray(wl.m[m_slice])
    if P_subset is not None:
        wl.P = np.ascontiguousarray(np.asarray(P_subset, dtype=np.uint32))
    if s_subset is not None:
        wl.s = np.ascontiguousarray(wl.s[s_subset])
    wl.sizes = np.ascontiguousarray(wl.sizes, dtype=np.float64)
    wl.gaps = np.ascontiguousarray(wl.gaps, dtype=np.float64)
    wl.L = np.ascontiguousarray(wl.L, dtype=np.float64)
    return wl


def make_measurements(wl, seed: int = 1):
    """Synthetic "measured" completion times for the scoring step, [n_ids, n_m, n_P], and the
    segment sizes they were taken with (same shape, uint32).  No model of the method enters:
    a plain positive curve in (strategy rank, m, P) with 20 % seeded noise, a constant offset
    and a delay of the small messages (the two error modes the paper reports), so that the
    arrays have the shape and scale of real ones.  seg: the largest power of two <= min(m, 8192)."""
    ids = [i for i in range(13) if (wl.strategy_mask >> i) & 1]
    m = np.asarray(wl.m, dtype=np.float64)
    P = np.asarray(wl.P, dtype=np.float64)
    rng = SplitMix64(408034000000 + 777 * seed)
    noise = rng.uniforms(len(ids) * m.size * P.size).reshape(len(ids), m.size, P.size)
    rank = (1.0 + np.arange(len(ids)) / 13.0)[:, None, None]
    base = (40.0 + m / 11.5)[None, :, None] * np.log2(P + 1.0)[None, None, :] * rank
    meas = base * (1.0 + 0.2 * noise) + 200.0
    meas = np.where(m[None, :, None] < 1024.0, meas * 1.5, meas)
    cap = np.minimum(np.asarray(wl.m, dtype=np.uint64), 8192)
    seg1 = (1 << (np.floor(np.log2(cap.astype(np.float64))).astype(np.uint64))).astype(np.uint32)
    seg = np.broadcast_to(seg1[None, :, None], meas.shape).copy()
    return meas, seg


def make_perturbed(wl: Workload, n_copies: int, eps: float, seed: int = 1) -> Workload:
    """A batch for the robustness check: table 0 of `wl` as it is, followed by n_copies copies in
    which every gap sample and the latency are scaled by independent factors uniform in
    [1 - eps, 1 + eps] (the sample sizes stay), over the same grid."""
    rng = SplitMix64(_seed(6) + 7919 * seed)
    n = wl.sizes.shape[1]
    u = rng.uniforms(n_copies * (n + 1)).reshape(n_copies, n + 1)
    f = 1.0 + eps * (2.0 * u - 1.0)
    sizes = np.repeat(wl.sizes[:1], n_copies + 1, axis=0)
    gaps = np.concatenate([wl.gaps[:1], wl.gaps[:1] * f[:, :n]], axis=0)
    L = np.concatenate([wl.L[:1], wl.L[0] * f[:, n]])
    return Workload(wl.name + "_perturbed", sizes, gaps, L, wl.m, wl.P, wl.s, wl.s_cap,
                    wl.strategy_mask, wl.dtype_size)
