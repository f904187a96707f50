/*
 * plogp.h -- C ABI of the MI355X (gfx950) pLogP collective-tuning library.
 *
 * The library evaluates the pLogP cost models of the Broadcast and Scatter
 * implementation strategies (paper: Table 1 and Table 2) over a grid of
 * message size m, process count P and segment size s, and for every (m, P)
 * keeps the predicted-fastest strategy and its best segment size (paper:
 * Section 3.1, the search of the segment size that minimises the predicted
 * time; Section 1, the choice of the most adapted technique per
 * (communication pattern, message size, number of processes)).
 *
 * Notation follows the paper's Section 2: g(m) is the gap of a message of m
 * bytes (a measured table), L the latency, P the number of nodes, s the
 * segment size, k the number of segments (here k = ceil(m / s)).
 *
 * Everything is computed by HIP kernels on the current HIP device; there is
 * no CPU fallback: without a usable GPU every compute entry point returns
 * PLOGP_EDEVICE.  All functions return a status (0 = PLOGP_OK), never throw,
 * never abort and never print.  Out-parameters are untouched on error.
 * Pointers are HOST pointers unless the name starts with d_ (DEVICE).
 * Calls that enqueue work take the HIP stream as a void* (hipStream_t; NULL
 * is the default stream) and are asynchronous with respect to the host unless
 * stated otherwise.  Handles may be used from one host thread at a time, and
 * belong to the device that was current when they were created: call with
 * that device current.
 *
 * Strategy ids (the order of the rows of Table 1, then Table 2):
 *    0 Broadcast flat tree                 7 Broadcast binomial tree
 *    1 Broadcast flat tree rendezvous      8 Broadcast binomial tree rendezvous
 *    2 Broadcast segmented flat tree       9 Broadcast segmented binomial tree
 *    3 Broadcast chain                    10 Scatter flat tree
 *    4 Broadcast chain rendezvous         11 Scatter chain
 *    5 Broadcast segmented chain          12 Scatter binomial tree
 *    6 Broadcast binary tree
 * Ids 2, 5 and 9 are the segmented rows (they take s); the others ignore s.
 *
 * Beyond the two tables (Section 3 names Gather and Barrier as patterns that are
 * built like Broadcast and Scatter; the paper prints no rows for them, these
 * follow from the same pLogP rules):
 *   13 Gather flat tree      (P-1) g(m) + L                      the rows of Table 2:
 *   14 Gather chain          sum_{j=1}^{P-1} g(j m) + (P-1) L    a Gather is its Scatter
 *   15 Gather binomial tree  sum_j g(2^j m) + ceil(log2 P) L     with every message reversed
 *   16 Barrier flat tree     2 ((P-1) g(1) + L)                  a one-byte fan-in to the root,
 *   17 Barrier binomial tree 2 (floor(log2 P) g(1) + ceil(log2 P) L)   then a one-byte fan-out
 * m of a Gather is the share of one process, as for Scatter; a Barrier ignores m.
 */
#ifndef PLOGP_H
#define PLOGP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PLOGP_N_STRATEGIES 18
#define PLOGP_MASK_BCAST 0x03FFu      /* ids 0..9  */
#define PLOGP_MASK_SCATTER 0x1C00u    /* ids 10..12 */
#define PLOGP_MASK_ALL 0x1FFFu        /* every row of Tables 1 and 2 */
#define PLOGP_MASK_GATHER 0xE000u     /* ids 13..15 */
#define PLOGP_MASK_BARRIER 0x30000u   /* ids 16, 17 */
#define PLOGP_MASK_EVERY 0x3FFFFu     /* ids 0..17 */
#define PLOGP_NO_STRATEGY 0xFFFFFFFFu
#define PLOGP_MAX_SAMPLES 4096        /* largest table that fits the LDS staging */
#define PLOGP_NO_CAP UINT64_MAX
#define PLOGP_MAX_TIME 6.668014432879854e+240  /* 2^800: largest gap or latency of a table */

enum {
    PLOGP_OK = 0,
    PLOGP_EINVAL = 1,   /* bad argument (see each function)                          */
    PLOGP_ERANGE = 2,   /* a size that enters a formula would reach 2^53, or a job   */
                        /* is too large for one launch                               */
    PLOGP_ENOSPC = 3,   /* output buffer too small                                   */
    PLOGP_ENOMEM = 4,   /* host or device allocation failed                          */
    PLOGP_EDEVICE = 5,  /* HIP error; plogp_last_hip_error() returns the HIP code    */
    PLOGP_ETOOBIG = 6   /* the job needs more scratch memory than the fixed buffer   */
                        /* of plogp_tune_grid_static holds                           */
};

/* One or several pLogP parameter tables {g(.), L}, resident on the device. */
typedef struct plogp_table plogp_table;
/* A tuning grid (m list, P list, s candidates), resident on the device. */
typedef struct plogp_grid plogp_grid;

/* One decision: what Section 1 of the paper selects per (pattern, m, P). */
typedef struct {
    double time;        /* predicted completion time of the chosen strategy        */
    uint32_t s;         /* chosen segment size in bytes, 0 = unsegmented           */
    uint32_t strategy;  /* chosen strategy id, PLOGP_NO_STRATEGY if none competed  */
} plogp_cell;           /* 16 bytes */

/* Caller-owned description of a grid; all arrays are host arrays. */
typedef struct {
    const uint64_t *m;      /* message sizes in bytes, > 0; duplicates allowed       */
    size_t n_m;
    const uint32_t *P;      /* process counts, >= 2, strictly ascending              */
    size_t n_P;
    const uint64_t *s;      /* segment-size candidates, > 0, < 2^32, strictly asc.   */
    size_t n_s;             /* may be 0 (then s may be NULL)                         */
    uint64_t s_cap;         /* a candidate competes for m iff s <= min(m, s_cap)     */
    uint32_t dtype_size;    /* m and s must be multiples of it (Section 2: s is a    */
                            /* multiple of the basic datatype); 0 or 1 = any         */
    uint32_t strategy_mask; /* bit i set = strategy id i competes                    */
} plogp_grid_desc;

/*
 * plogp_load_table / plogp_load_tables -- paper Section 2 (the measured g(m)
 * and L that feed the models).  Copies n_tables tables of n samples each to
 * the device and computes there the slope of every interval between samples
 * (g between samples is read as piecewise linear; below the first sample it is
 * clamped to the first gap, above the last sample the last line continues).
 *   sizes [n_tables][n]: sample sizes in bytes, integers in [1, 2^53), strictly
 *                        increasing within a table;
 *   gaps  [n_tables][n]: g at those sizes, in [0, PLOGP_MAX_TIME] (need not be monotone);
 *   L     [n_tables]   : latency, in [0, PLOGP_MAX_TIME];
 *                        (with this bound no model value can overflow: a predicted time is
 *                        +infinity only where no segment size competes)
 *   2 <= n <= PLOGP_MAX_SAMPLES, n_tables >= 1.
 * Synchronous.  Inputs are copied; the handle owns host and device copies and
 * is released with plogp_free_table.  Errors: EINVAL, ENOMEM, EDEVICE.
 */
int plogp_load_table(const double *sizes, const double *gaps, size_t n, double L,
                     plogp_table **out);
int plogp_load_tables(const double *sizes, const double *gaps, size_t n, const double *L,
                      size_t n_tables, plogp_table **out);
int plogp_free_table(plogp_table *t);
size_t plogp_table_count(const plogp_table *t);
size_t plogp_table_samples(const plogp_table *t);
/* Reads back the device-computed interval slopes of one table (n doubles;
 * slope[n-1] repeats slope[n-2]).  Synchronous.  For tests. */
int plogp_table_slopes(const plogp_table *t, size_t table_index, double *slopes_out, size_t n);

/*
 * plogp_interp_g -- paper Section 2, g(z): the gap of table `table_index`
 * at n arbitrary sizes.  d_z: n device uint64 (each in [1, 2^53)); d_g_out: n
 * device doubles.  Enqueued on `stream`.  n = 0 is a no-op.
 * Errors: EINVAL (null, bad index), EDEVICE.  Values of d_z are not checked.
 */
int plogp_interp_g(const plogp_table *t, size_t table_index, const uint64_t *d_z, size_t n,
                   double *d_g_out, void *stream);

/*
 * plogp_eval_strategy -- paper Table 1 / Table 2: the predicted time of ONE
 * strategy at n independent points (m, P, s) on table `table_index`.
 *   d_m [n] uint64 bytes, > 0; d_P [n] uint32, >= 2; d_s [n] uint64 segment
 *   sizes (only read for ids 2, 5, 9, where 0 < s <= m; may be NULL for
 *   the other ids); d_time_out [n] doubles.  All device pointers.  Ids 13..17
 *   (Gather, Barrier: see the list of ids above) are evaluated the same way.
 * A point outside the domain (m = 0, P < 2, bad s, or a product j*m that
 * would reach 2^53) yields NaN for that point.  Enqueued on `stream`.
 * Errors: EINVAL (null pointers, unknown strategy, bad index), EDEVICE.
 */
int plogp_eval_strategy(const plogp_table *t, size_t table_index, int strategy,
                        const uint64_t *d_m, const uint32_t *d_P, const uint64_t *d_s,
                        size_t n, double *d_time_out, void *stream);

/*
 * plogp_grid_create -- validates a grid and makes it resident on the device.
 * Synchronous.  The description and its arrays are copied.
 * Errors: EINVAL (null array with non-zero count; n_m = 0 or n_P = 0; m = 0;
 *         P < 2 or not strictly ascending; s = 0, s >= 2^32 or not strictly
 *         ascending; m or s not a multiple of dtype_size; mask selects no
 *         known strategy), ERANGE (m >= 2^53, or with a Scatter or Gather chain /
 *         binomial row enabled (Pmax-1)*m_max or 2^(ceil(log2 Pmax)-1)*m_max >= 2^53),
 *         ENOMEM, EDEVICE.
 */
int plogp_grid_create(const plogp_grid_desc *desc, plogp_grid **out);
int plogp_grid_free(plogp_grid *g);

/* Number of operation planes of the decision table: Broadcast if any of ids
 * 0..9 is in the mask, then Scatter (10..12), Gather (13..15), Barrier (16, 17),
 * each if any of its ids is: 1 to 4. */
size_t plogp_grid_ops(const plogp_grid *g);
/* Cells / bytes of the decision table for n_tables tables over this grid (0 for a null grid,
 * and if the byte count would not fit a size_t). */
size_t plogp_decision_table_cells(size_t n_tables, const plogp_grid *g);
size_t plogp_decision_table_bytes(size_t n_tables, const plogp_grid *g);

/*
 * plogp_tune_grid -- the whole sweep (paper Section 3.1 and Section 1): for
 * every table of `t`, every operation plane and every (m, P) of the grid,
 * evaluates all enabled strategies (segmented ones for every candidate
 * s <= min(m, s_cap)) and writes the arg-min: smallest predicted time, ties
 * to the lowest strategy id, then to the smallest s.  The operations (Broadcast,
 * Scatter, Gather, Barrier) never compete with each other: each has a plane.
 *   d_out: DEVICE buffer, caller-owned, 16-byte aligned, laid out
 *          [table][operation plane][m index][P index] with P fastest;
 *          d_out_bytes must be >= plogp_decision_table_bytes().
 * A cell in which no strategy competed (e.g. only segmented ids enabled and
 * no candidate <= m) is {+inf, 0, PLOGP_NO_STRATEGY}.
 * Enqueued on `stream`; the result is complete when the stream reaches this
 * point.  Scratch memory is owned by the grid handle (one block, allocated on
 * first use, replaced only when a later call needs a larger one): two calls
 * that use the same grid handle's scratch (plogp_tune_grid, plogp_score_grid)
 * must not overlap.  The table handle is only read.
 * Errors: EINVAL (null, misaligned d_out), ENOSPC, ERANGE (the job would need a
 * launch of 2^31 workgroups or more: split the batch or the grid), ENOMEM,
 * EDEVICE.
 */
int plogp_tune_grid(const plogp_table *t, plogp_grid *g, plogp_cell *d_out, size_t d_out_bytes,
                    void *stream);

/*
 * Cut-over extraction -- paper Section 3.1 (how the tuned segment size is
 * applied: messages above some size are segmented, smaller ones are not) and
 * Section 1 (one technique per pattern, message size and node count): every
 * row of a decision table -- the cells of one (table, operation, P) read along
 * the grid's message sizes in their given order -- is compressed into its runs
 * of equal decision.  A run starts at the first cell of a row and at every
 * cell whose key differs from the key of the cell before it; the key is the
 * strategy id (PLOGP_KEY_STRATEGY) or the pair (strategy id, s)
 * (PLOGP_KEY_STRATEGY_AND_SEGMENT).  A run is reported by its first cell.
 */
#define PLOGP_KEY_STRATEGY 0
#define PLOGP_KEY_STRATEGY_AND_SEGMENT 1

typedef struct {
    uint64_t m_from;    /* message size of the first cell of the run               */
    uint32_t s;         /* that cell's segment size, 0 = unsegmented               */
    uint32_t strategy;  /* that cell's strategy id                                  */
} plogp_run;            /* 16 bytes */

/* Rows of the decision table of n_tables tables over this grid:
 * n_tables * operation planes * process counts, ordered (table, operation, P). */
size_t plogp_cutover_rows(size_t n_tables, const plogp_grid *g);

/*
 * plogp_cutovers -- extracts the runs of a decision table that is laid out as
 * plogp_tune_grid writes it for n_tables tables over grid g.
 *   d_cells:       DEVICE, the decision table, 16-byte aligned (read only);
 *   d_row_offsets: DEVICE, plogp_cutover_rows() + 1 uint64: the runs of row r
 *                  are d_runs[d_row_offsets[r] .. d_row_offsets[r+1]); the last
 *                  entry is the total number of runs;
 *   d_runs:        DEVICE, room for runs_capacity records, 16-byte aligned,
 *                  ordered by row, then by message-size index.  Runs whose
 *                  index is >= runs_capacity are not written (the offsets and
 *                  the total still are): the caller compares the total with
 *                  its capacity.  plogp_decision_table_cells() records always
 *                  suffice.  May be NULL when runs_capacity is 0 (count only).
 * Enqueued on `stream`.  Scratch is owned by the grid handle (allocated on
 * first use): two extractions on one grid handle must not overlap.
 * Errors: EINVAL (null, misaligned, bad key_mode, n_tables = 0), ERANGE (more
 * than 2^36 (row, 16 sizes) pieces), ENOMEM, EDEVICE.
 */
int plogp_cutovers(plogp_grid *g, size_t n_tables, const plogp_cell *d_cells, int key_mode,
                   uint64_t *d_row_offsets, plogp_run *d_runs, size_t runs_capacity, void *stream);

/*
 * Prediction against measurement -- paper Section 4: every implementation is
 * measured, the measured completion times are set against the predictions of
 * Tables 1 and 2, and the question is whether the technique the models choose
 * is the fastest one in the measurement.  For ONE table and the (m, P) of grid
 * g (its candidate list and cap are not used), with r running over the
 * strategies of Tables 1 and 2 (ids 0..12; the paper measures no other) that are
 * enabled in the grid's mask, in ascending id:
 *   pred[r][m][P]     the model at the measured point;
 *   verdict[op][m][P] pred_best: the enabled strategy of the operation with the
 *                     smallest prediction; meas_best: the one with the smallest
 *                     measured time (ties to the lowest id in both);
 *                     regret = meas[pred_best] / meas[meas_best] - 1, i.e. 0
 *                     when the decision survives;
 *   scores[r]         over all (m, P): e = |(pred - meas) / meas|: count,
 *                     maximum, and sum (added per m in ascending P, then over
 *                     ascending m, so that it is reproducible bit for bit).
 */
typedef struct {
    double regret;       /* how much slower the predicted choice was measured  */
    uint32_t pred_best;  /* strategy id with the smallest prediction           */
    uint32_t meas_best;  /* strategy id with the smallest measured time        */
} plogp_verdict;         /* 16 bytes */

typedef struct {
    double sum_abs_err;  /* sum of |(pred - meas) / meas|                      */
    double max_abs_err;  /* its maximum                                        */
    uint64_t count;      /* points                                             */
    uint64_t reserved;   /* 0                                                  */
} plogp_strategy_score;  /* 32 bytes */

/* Strategies with ids 0..12 enabled in the grid's mask: the rows of meas, seg, pred, scores. */
size_t plogp_score_strategies(const plogp_grid *g);

/*
 * plogp_score_grid -- all DEVICE pointers:
 *   d_meas    [rows][n_m][n_P] doubles, measured times (> 0);
 *   d_seg     [rows][n_m][n_P] uint32, the segment size each point was measured
 *             with; read for ids 2, 5, 9 only (0 < s <= m, else the prediction
 *             is NaN: it is never pred_best, the maximum skips it and that
 *             strategy's sum becomes NaN); may be NULL when none of them is
 *             enabled;
 *   d_pred    [rows][n_m][n_P] doubles (out);
 *   d_verdict [operation planes][n_m][n_P] records (out), planes as in
 *             plogp_tune_grid, 16-byte aligned;
 *   d_scores  [rows] records (out), 16-byte aligned.
 * Enqueued on `stream`.  Uses the grid handle's scratch like plogp_tune_grid:
 * calls on one grid handle must not overlap.
 * Errors: EINVAL (null, misaligned, bad table index), ENOMEM, EDEVICE.
 */
int plogp_score_grid(const plogp_table *t, size_t table_index, plogp_grid *g, const double *d_meas,
                     const uint32_t *d_seg, double *d_pred, plogp_verdict *d_verdict,
                     plogp_strategy_score *d_scores, void *stream);

/*
 * Decision robustness -- paper Section 4 and the conclusion: the deviations
 * between prediction and reality did not change which technique the models
 * select.  For a batch of n_tables decision tables over grid g, laid out as
 * plogp_tune_grid writes them ([table][operation plane][m][P]), table 0 tuned
 * from the parameters as measured and tables 1.. from perturbed copies:
 *   d_agree       [planes][n_m][n_P] uint32 (out): how many of the tables 1..
 *                 hold the decision of table 0 in that cell (the fraction that
 *                 keeps it is d_agree / (n_tables - 1));
 *   d_max_dev     same shape, doubles (out), or NULL: the largest
 *                 abs(T_t - T_0) / T_0 of the cell's predicted time over those
 *                 tables (0 for one table; a NaN quotient is skipped);
 *   d_table_agree [n_tables] uint32 (out), or NULL: in how many cells table t
 *                 holds the decision of table 0 (entry 0 = number of cells).
 * key_mode as in plogp_cutovers: the decision is the strategy, or the strategy
 * and its segment size.  All DEVICE pointers; d_cells 16-byte aligned.
 * Enqueued on `stream`; uses no scratch memory.
 * Errors: EINVAL (null, misaligned, bad key_mode, n_tables = 0 or above 2^24),
 * ERANGE (more than 2^32 - 256 cells per table), EDEVICE.
 */
int plogp_robustness(const plogp_grid *g, size_t n_tables, const plogp_cell *d_cells, int key_mode,
                     uint32_t *d_agree, double *d_max_dev, uint32_t *d_table_agree, void *stream);

/*
 * plogp_tune_grid_static -- plogp_tune_grid for callers that cannot allocate:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same result, same kernels; but the scratch memory
 * of the kernels (the per-size and per-candidate terms, the Scatter-chain block
 * sums, the tables turned round for a batch) is not taken from the grid handle:
 * it is a fixed buffer of PLOGP_STATIC_SCRATCH_BYTES inside the library's code
 * object, one per GPU, held until the process ends.  The call allocates and
 * frees nothing and does not wait for the device.  A job whose scratch does not
 * fit the buffer is refused with PLOGP_ETOOBIG before anything is launched (use
 * plogp_tune_grid, or split the batch or the grid).  The grid handle is only
 * read, so it may be shared with a plogp_tune_grid call in flight.
 * Every call on one GPU uses that GPU's one buffer, whatever the handles and
 * streams: calls that overlap on one GPU race; calls on one stream, or ordered
 * by events, do not.  No kernel reads scratch it has not written in the same
 * call, so nothing is cleared between calls.
 * The buffer's address is looked up once per GPU (at the library's first call on
 * that GPU, a table load or grid creation included), with that GPU current.
 * Errors: as plogp_tune_grid, plus ETOOBIG; never ENOMEM.
 */
#define PLOGP_STATIC_SCRATCH_BYTES (64u << 20)
int plogp_tune_grid_static(const plogp_table *t, const plogp_grid *g, plogp_cell *d_out,
                           size_t d_out_bytes, void *stream);

/* Message for a status code (static string). */
const char *plogp_strerror(int status);
/* HIP error code of the calling thread's most recent PLOGP_EDEVICE (0 if none). */
int plogp_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PLOGP_H */
