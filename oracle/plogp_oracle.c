/*
 * plogp_oracle.c -- plain CPU oracle for the pLogP tuning sweep.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the referee the HIP library is
 * checked against and the CPU baseline the benchmark times beside it.  It
 * shares no code with the HIP library; nothing in the product path may call
 * it.  It is written to be checked against the paper by eye, not to be fast.
 *
 * What it computes (paper: Section 2 for g(m), L, P, s, k; Table 1 for the
 * ten Broadcast models, Table 2 for the three Scatter models; Section 3.1
 * for the search of the segment size that minimises the predicted time and
 * the choice of the predicted-fastest strategy per (pattern, m, P)):
 *
 *   for every (table, operation, m, P):
 *       best = +inf
 *       for strategy id ascending:                 (ids in table order, 0..12; then the
 *                                                   Gather rows 13..15 and Barrier rows 16, 17
 *                                                   that Section 3 says are built alike)
 *           unsegmented: T = model(id, m, P);      keep on strict T < best
 *           segmented:   for s ascending, s <= min(m, s_cap):
 *                            T = model(id, m, P, s); keep on strict T < best
 *       cell = (best T, best s or 0, best id)
 *
 * Arithmetic: IEEE binary64, round to nearest even, no contraction (build
 * with -ffp-contract=off); fma() only where written.  All integers that
 * enter a formula (m, s, k, P-1, floor/ceil log2 P, j*m, 2^j*m) are exact in
 * binary64 (callers keep them below 2^53).
 *
 * Readings of points the paper leaves open (each is a convention):
 *   - g between samples: piecewise linear; below the first sample: clamped to
 *     the first gap; above the last sample: the last interval's line goes on.
 *   - k = ceil(m / s)  (the paper says "k segments"; with s | m this equals
 *     its floor(m/s)).
 *   - Binary tree: the printed bound is evaluated as an equality.
 *   - floor(log2 P), ceil(log2 P): integer arithmetic, as printed.
 *   - Sum over j of g(j*m) in the Scatter chain row: blocks of 64 consecutive
 *     j starting at j = 1; a running sum inside the block, block totals added
 *     in ascending order.  For P <= 65 this is plain left-to-right summation.
 *   - Sum over j of g(2^j*m): plain left-to-right.
 *   - Ties: lowest strategy id, then smallest s (strict '<' in ascending
 *     order gives exactly that).
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * (exact-arithmetic tables with integer closed forms, an event simulator
 * that replays the send/receive schedules, structural ties, rational
 * re-evaluation of every rounding, brute force on tiny grids, the convex
 * optimum of the segmented chain on affine g, metamorphic scaling).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    double time;
    uint32_t s;
    uint32_t strategy;
} oracle_cell;

typedef struct {
    const double *x;      /* sample sizes, strictly increasing            */
    const double *y;      /* gap samples                                  */
    double *slope;        /* slope[i] of interval [x[i], x[i+1]]          */
    size_t n;
    double L;
} oracle_table;

#define N_STRATEGIES 18       /* Table 1 (0..9), Table 2 (10..12), Gather (13..15), Barrier (16, 17) */
#define SUM_BLOCK 64

/* ---- g(): Section 2 defines g(m); the evaluation rule between samples is
 *      piecewise-linear interpolation ------------------------------------- */

void plogp_oracle_slopes(const double *x, const double *y, size_t n, double *slope)
{
    for (size_t i = 0; i + 1 < n; ++i) {
        double dy = y[i + 1] - y[i];
        double dx = x[i + 1] - x[i];
        slope[i] = dy / dx;
    }
    slope[n - 1] = slope[n - 2];
}

/* index of the last sample with x <= z, clamped to [0, n-1] */
static size_t interval_of(const double *x, size_t n, double z)
{
    size_t lo = 0, hi = n;            /* first index with x > z, by bisection */
    while (lo < hi) {
        size_t mid = lo + (hi - lo) / 2;
        if (x[mid] <= z)
            lo = mid + 1;
        else
            hi = mid;
    }
    return lo == 0 ? 0 : lo - 1;
}

static double gap(const oracle_table *t, double z)
{
    size_t i = interval_of(t->x, t->n, z);
    double zc = z > t->x[0] ? z : t->x[0];
    double d = zc - t->x[i];
    return fma(t->slope[i], d, t->y[i]);
}

double plogp_oracle_g(const double *x, const double *y, size_t n, double z)
{
    oracle_table t;
    t.x = x; t.y = y; t.n = n; t.L = 0.0;
    t.slope = (double *)malloc(n * sizeof(double));
    plogp_oracle_slopes(x, y, n, t.slope);
    double g = gap(&t, z);
    free(t.slope);
    return g;
}

/* ---- integer terms of Tables 1 and 2 ------------------------------------ */

static unsigned floor_log2(uint32_t P)
{
    unsigned f = 0;
    while ((P >> (f + 1)) != 0)
        ++f;
    return f;
}

static unsigned ceil_log2(uint32_t P)
{
    unsigned f = floor_log2(P);
    return ((uint32_t)1 << f) == P ? f : f + 1;
}

/* ---- the two sums of Table 2 -------------------------------------------- */

/* sum_{j=1}^{P-1} g(j*m), blocked association order */
static double scatter_chain_sum(const oracle_table *t, uint64_t m, uint32_t P)
{
    double done = 0.0;       /* total of the finished blocks */
    double run = 0.0;        /* running sum inside the current block */
    for (uint32_t j = 1; j <= P - 1; ++j) {
        run = run + gap(t, (double)((uint64_t)j * m));
        if (j % SUM_BLOCK == 0) {
            done = done + run;
            run = 0.0;
        }
    }
    return done + run;
}

/* the same sum for every P = 2..Pmax in one pass over j: out[P] */
static void scatter_chain_prefix(const oracle_table *t, uint64_t m, uint32_t Pmax, double *out)
{
    double done = 0.0, run = 0.0;
    for (uint32_t j = 1; j <= Pmax - 1; ++j) {
        run = run + gap(t, (double)((uint64_t)j * m));
        if (j % SUM_BLOCK == 0) {
            done = done + run;
            run = 0.0;
        }
        out[j + 1] = done + run;
    }
}

/* sum_{j=0}^{ceil(log2 P)-1} g(2^j * m), left to right */
static double scatter_binomial_sum(const oracle_table *t, uint64_t m, uint32_t P)
{
    unsigned cl = ceil_log2(P);
    double sum = 0.0;
    for (unsigned j = 0; j < cl; ++j)
        sum = sum + gap(t, (double)(m << j));
    return sum;
}

/* ---- the thirteen models -------------------------------------------------
 * chain_sum: value of sum_j g(j*m) for this (m, P) if the caller already has
 * it, NaN to have it computed here.                                          */
static double model(const oracle_table *t, int id, uint64_t m, uint32_t P, uint64_t s,
                    double chain_sum)
{
    const double L = t->L;
    const double q = (double)(P - 1);
    const double fl = (double)floor_log2(P);
    const double cl = (double)ceil_log2(P);
    const double gm = gap(t, (double)m);
    const double g1 = gap(t, 1.0);
    const double R = fma(3.0, L, 2.0 * g1);           /* 2 g(1) + 3 L */
    double gs = 0.0, k = 0.0;
    if (id == 2 || id == 5 || id == 9) {
        gs = gap(t, (double)s);
        k = (double)((m + s - 1) / s);                /* k = ceil(m / s) */
    }
    switch (id) {
    /* Table 1, Broadcast */
    case 0:  return fma(q, gm, L);                    /* (P-1) g(m) + L                       */
    case 1:  return fma(q, gm, R);                    /* (P-1) g(m) + 2 g(1) + 3 L            */
    case 2:  return fma(q, gs * k, L);                /* (P-1) (g(s) k) + L                   */
    case 3:  return q * (gm + L);                     /* (P-1) (g(m) + L)                     */
    case 4:  return q * (gm + R);                     /* (P-1) (g(m) + 2 g(1) + 3 L)          */
    case 5:  return fma(q, gs + L, gs * (k - 1.0));   /* (P-1) (g(s) + L) + g(s) (k-1)        */
    case 6:  return cl * fma(2.0, gm, L);             /* ceil(log2 P) (2 g(m) + L)            */
    case 7:  return fma(fl, gm, cl * L);              /* floor(log2 P) g(m) + ceil(log2 P) L  */
    case 8:  return fma(fl, gm, cl * R);              /* ... + ceil(log2 P) (2 g(1) + 3 L)    */
    case 9:  return fma(fl, gs * k, cl * L);          /* floor(log2 P) g(s) k + ceil(log2 P) L*/
    /* Table 2, Scatter (m is the share of one process) */
    case 10: return fma(q, gm, L);                    /* (P-1) g(m) + L                       */
    case 11: {
        double sum = isnan(chain_sum) ? scatter_chain_sum(t, m, P) : chain_sum;
        return fma(q, L, sum);                        /* sum_j g(j m) + (P-1) L               */
    }
    case 12: return fma(cl, L, scatter_binomial_sum(t, m, P)); /* sum_j g(2^j m) + ceil(log2 P) L */
    /* Gather (Section 3 names it as built like these): a Scatter read backwards.  Every
     * message of Table 2's schedules travels the other way, at the other end of the same
     * time span, and the root's receptions are one gap apart as its sends were: the same
     * three expressions, m again the share of one process. */
    case 13: return fma(q, gm, L);                    /* flat: the root takes in P-1 shares   */
    case 14: {
        double sum = isnan(chain_sum) ? scatter_chain_sum(t, m, P) : chain_sum;
        return fma(q, L, sum);                        /* chain: the shares pile up hop by hop */
    }
    case 15: return fma(cl, L, scatter_binomial_sum(t, m, P)); /* binomial: subtrees merge    */
    /* Barrier (Section 3, likewise): no payload; a one-byte fan-in to the root followed by
     * a one-byte fan-out.  Flat: each half is the flat-tree row of Table 1 with g(1);
     * binomial: each half is its binomial-tree row with g(1).  m is not used. */
    case 16: return 2.0 * fma(q, g1, L);              /* 2 ((P-1) g(1) + L)                   */
    case 17: return 2.0 * fma(fl, g1, cl * L);        /* 2 (floor(log2 P) g(1) + ceil(log2 P) L) */
    default: return NAN;
    }
}

static int is_segmented(int id) { return id == 2 || id == 5 || id == 9; }

/* One model value.  s is ignored for unsegmented ids.  Returns 0, or -1 on
 * arguments outside the model's domain. */
int plogp_oracle_eval(const double *x, const double *y, size_t n, double L, int id,
                      uint64_t m, uint32_t P, uint64_t s, double *out)
{
    if (n < 2 || id < 0 || id >= N_STRATEGIES || P < 2 || m == 0)
        return -1;
    if (is_segmented(id) && (s == 0 || s > m))
        return -1;
    oracle_table t;
    t.x = x; t.y = y; t.n = n; t.L = L;
    t.slope = (double *)malloc(n * sizeof(double));
    plogp_oracle_slopes(x, y, n, t.slope);
    *out = model(&t, id, m, P, s, NAN);
    free(t.slope);
    return 0;
}

/* arg-min over the strategies lo..hi of one operation for one (m, P) */
static oracle_cell best_of(const oracle_table *t, int lo, int hi, uint32_t mask,
                           uint64_t m, uint32_t P, const uint64_t *s, size_t n_s,
                           uint64_t s_cap, double chain_sum)
{
    oracle_cell c;
    c.time = INFINITY; c.s = 0; c.strategy = 0xFFFFFFFFu;
    uint64_t limit = m < s_cap ? m : s_cap;
    for (int id = lo; id <= hi; ++id) {
        if (!((mask >> id) & 1u))
            continue;
        if (!is_segmented(id)) {
            double T = model(t, id, m, P, 0, chain_sum);
            if (T < c.time) { c.time = T; c.s = 0; c.strategy = (uint32_t)id; }
        } else {
            for (size_t i = 0; i < n_s; ++i) {
                if (s[i] > limit)
                    continue;
                double T = model(t, id, m, P, s[i], chain_sum);
                if (T < c.time) { c.time = T; c.s = (uint32_t)s[i]; c.strategy = (uint32_t)id; }
            }
        }
    }
    return c;
}

/*
 * Decision tables for a batch of tables over one grid.
 * x, y: [n_tables][n]; L: [n_tables]; out: [n_tables][n_ops][n_m][n_P] with P
 * fastest, where the operations present are Broadcast (if any id 0..9 is in
 * mask), then Scatter (10..12), Gather (13..15), Barrier (16, 17).  Naive per cell, except that the
 * Scatter-chain sum is produced once per (table, m) for all P.
 * Returns the number of threads used, or -1 on a bad argument.
 */
int plogp_oracle_tune(const double *x, const double *y, size_t n, const double *L,
                      size_t n_tables, const uint64_t *m, size_t n_m, const uint32_t *P,
                      size_t n_P, const uint64_t *s, size_t n_s, uint64_t s_cap,
                      uint32_t mask, oracle_cell *out, int n_threads)
{
    if (n < 2 || n_tables == 0 || n_m == 0 || n_P == 0)
        return -1;
    /* the operations present, in plane order: Broadcast, Scatter, Gather, Barrier */
    static const int op_lo[4] = {0, 10, 13, 16}, op_hi[4] = {9, 12, 15, 17};
    int has_op[4];
    size_t n_ops = 0;
    for (int op = 0; op < 4; ++op) {
        has_op[op] = 0;
        for (int id = op_lo[op]; id <= op_hi[op]; ++id)
            if ((mask >> id) & 1u) has_op[op] = 1;
        n_ops += (size_t)has_op[op];
    }
    uint32_t Pmax = 0;
    for (size_t i = 0; i < n_P; ++i) {
        if (P[i] < 2) return -1;
        if (P[i] > Pmax) Pmax = P[i];
    }
    int used = 1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
    #pragma omp parallel
    {
        #pragma omp single
        used = omp_get_num_threads();
    }
#endif
    (void)n_threads;
    const long long n_rows = (long long)(n_tables * n_m);
    #pragma omp parallel
    {
        double *slope = (double *)malloc(n * sizeof(double));
        double *chain = (double *)malloc(((size_t)Pmax + 2) * sizeof(double));
        #pragma omp for schedule(dynamic, 1)
        for (long long row = 0; row < n_rows; ++row) {
            const size_t ti = (size_t)row / n_m, mi = (size_t)row % n_m;
            oracle_table t;
            t.x = x + ti * n; t.y = y + ti * n; t.n = n; t.L = L[ti]; t.slope = slope;
            plogp_oracle_slopes(t.x, t.y, n, slope);
            const int need_chain = ((mask >> 11) & 1u) | ((mask >> 14) & 1u);
            if (need_chain)
                scatter_chain_prefix(&t, m[mi], Pmax, chain);
            for (size_t pi = 0; pi < n_P; ++pi) {
                const double cs = need_chain ? chain[P[pi]] : 0.0;
                size_t plane = 0;
                for (int op = 0; op < 4; ++op) {
                    if (!has_op[op])
                        continue;
                    out[((ti * n_ops + plane) * n_m + mi) * n_P + pi] =
                        best_of(&t, op_lo[op], op_hi[op], mask, m[mi], P[pi], s, n_s, s_cap, cs);
                    ++plane;
                }
            }
        }
        free(slope);
        free(chain);
    }
    return used;
}

/* ---- prediction against measurement ---------------------------------------
 *
 * The step after the tuning in the paper (Section 4): each implementation is
 * measured, the measured completion times are set against the model's
 * predictions, and the question is whether the technique the models choose
 * is the one that is fastest in the measurement.  Here, for one table and a
 * grid of (m, P), with `meas` the measured time of every enabled strategy at
 * every (m, P) and `seg` the segment size it was measured with (read for the
 * segmented ids 2, 5, 9 only; 0 < s <= m):
 *
 *   pred[r][m][P]     the model at the measured point (r: rank of the strategy
 *                     id among the enabled ones, ascending)
 *   verdict[op][m][P] pred_best = the enabled strategy of the operation with
 *                     the smallest prediction, meas_best = the one with the
 *                     smallest measured time (strict '<' in ascending id: ties
 *                     to the lowest id), regret = meas[pred_best] /
 *                     meas[meas_best] - 1 (0 when the decision survives)
 *   score[r]          over all (m, P): e = |(pred - meas) / meas|; count;
 *                     max e; sum e, added per m in ascending P from +0.0 and
 *                     the per-m sums added in ascending m from +0.0
 *
 * Operations present as in plogp_oracle_tune.  Returns 0, or -1 on a bad
 * argument.
 */
typedef struct {
    double regret;
    uint32_t pred_best;
    uint32_t meas_best;
} oracle_verdict;

typedef struct {
    double sum_abs_err;
    double max_abs_err;
    uint64_t count;
    uint64_t reserved;
} oracle_score;

int plogp_oracle_score(const double *x, const double *y, size_t n, double L, const uint64_t *m,
                       size_t n_m, const uint32_t *P, size_t n_P, uint32_t mask,
                       const double *meas, const uint32_t *seg, double *pred,
                       oracle_verdict *verdict, oracle_score *score)
{
    if (n < 2 || n_m == 0 || n_P == 0 || (mask & 0x1FFFu) == 0)
        return -1;
    mask &= 0x1FFFu;
    int ids[N_STRATEGIES], n_ids = 0;
    for (int id = 0; id < 13; ++id)                  /* the measured rows are those of Tables 1 and 2 */
        if ((mask >> id) & 1u)
            ids[n_ids++] = id;
    const int has_b = (mask & 0x3FFu) != 0;
    oracle_table t;
    double *slope = (double *)malloc(n * sizeof(double));
    t.x = x; t.y = y; t.n = n; t.L = L; t.slope = slope;
    plogp_oracle_slopes(x, y, n, slope);
    const size_t plane = n_m * n_P;
    for (size_t mi = 0; mi < n_m; ++mi) {
        for (size_t pi = 0; pi < n_P; ++pi) {
            if (P[pi] < 2 || m[mi] == 0) { free(slope); return -1; }
            for (int r = 0; r < n_ids; ++r) {
                const size_t at = (size_t)r * plane + mi * n_P + pi;
                const uint64_t s = is_segmented(ids[r]) ? seg[at] : 0;
                if (is_segmented(ids[r]) && (s == 0 || s > m[mi])) { free(slope); return -1; }
                pred[at] = model(&t, ids[r], m[mi], P[pi], s, NAN);
            }
            for (int op = 0; op < 2; ++op) {
                const int lo = op == 0 ? 0 : 10, hi = op == 0 ? 9 : 12;
                double best_p = INFINITY, best_m = INFINITY, meas_of_pred_best = NAN;
                uint32_t id_p = 0xFFFFFFFFu, id_m = 0xFFFFFFFFu;
                int any = 0;
                for (int r = 0; r < n_ids; ++r) {
                    if (ids[r] < lo || ids[r] > hi)
                        continue;
                    any = 1;
                    const size_t at = (size_t)r * plane + mi * n_P + pi;
                    if (pred[at] < best_p) { best_p = pred[at]; id_p = (uint32_t)ids[r]; meas_of_pred_best = meas[at]; }
                    if (meas[at] < best_m) { best_m = meas[at]; id_m = (uint32_t)ids[r]; }
                }
                if (!any)
                    continue;
                oracle_verdict *v = verdict + (size_t)(op == 0 ? 0 : has_b) * plane + mi * n_P + pi;
                v->pred_best = id_p;
                v->meas_best = id_m;
                v->regret = meas_of_pred_best / best_m - 1.0;
            }
        }
    }
    for (int r = 0; r < n_ids; ++r) {
        double total = 0.0, worst = 0.0;
        for (size_t mi = 0; mi < n_m; ++mi) {
            double row = 0.0;
            for (size_t pi = 0; pi < n_P; ++pi) {
                const size_t at = (size_t)r * plane + mi * n_P + pi;
                const double e = fabs((pred[at] - meas[at]) / meas[at]);
                row = row + e;
                if (e > worst) worst = e;
            }
            total = total + row;
        }
        score[r].sum_abs_err = total;
        score[r].max_abs_err = worst;
        score[r].count = (uint64_t)plane;
        score[r].reserved = 0;
    }
    free(slope);
    return 0;
}
