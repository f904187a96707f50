// Internal interface between the C-ABI host layer (plogp_api.hip) and the
// gfx950 kernels (plogp_kernels.hip).  Not installed; include/plogp.h is the
// public boundary.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace plogp {

// Number of consecutive terms j summed by one lane in the Scatter-chain sum
// (Table 2, chain row).  The association order of that sum is: blocks of
// SUM_BLOCK consecutive j starting at j = 1, a running sum inside a block,
// block totals added in ascending block order.
constexpr int SUM_BLOCK = 64;

// Most candidates s for which the sweeps that keep s in a lane's loop are used
// (more: the sweep that runs its lanes over s).
constexpr int SWEEP_M_MAX_S = 256;

// Device-resident batch of tables.
struct DeviceTables {
    const double *x;      // [n_tables][n] sample sizes
    const double *y;      // [n_tables][n] gaps
    const double *slope;  // [n_tables][n] interval slopes (written once, when the tables are loaded)
    const double *L;      // [n_tables]
    int n;                // samples per table
    int n_tables;
    int shared_x;         // 1: every table has the sample sizes of table 0
};

// Device-resident grid plus the index metadata of the Scatter-chain blocks.
struct DeviceGrid {
    const uint64_t *m;    // [n_m]
    const uint64_t *mu;   // [n_mu] the distinct message sizes, ascending (the Scatter-chain sums are
                          //        formed once per distinct size)
    const int *m_map;     // [n_m] index into mu of each message size
    const uint32_t *P;    // [n_P] strictly ascending
    const uint64_t *s;    // [n_s] strictly ascending
    const int *blk_off;   // [n_blk + 1] P-index range whose (P-1)/SUM_BLOCK equals the block
    const unsigned long long *blk_mask;  // [n_blk] bit r set: a grid P has P-1 == SUM_BLOCK*b + r
    int n_m, n_P, n_s;
    int n_mu;
    int n_blk;            // (Pmax-1)/SUM_BLOCK + 1 blocks; the last one may be partial
    int last_terms;       // number of terms of the last block: (Pmax-1) - SUM_BLOCK*(n_blk-1)
    int cl_max;           // ceil(log2 Pmax)
    uint64_t s_cap;
    uint32_t mask;        // which rows of Tables 1 and 2 compete (bits 0..12)
    uint32_t extra;       // rows beyond the tables: bits 0..2 Gather flat / chain / binomial (ids 13..15),
                          // bits 3, 4 Barrier flat / binomial (ids 16, 17)
    uint32_t need;        // bit 11: the sums over j of g(j m) are wanted, bit 12: those of g(2^j m)
                          // (by a Scatter row or by its Gather twin)
    int n_ops;            // planes of the decision table: Broadcast, Scatter, Gather, Barrier, those present
    int blk_is_prefix;    // 1: a kernel turns the block totals into their exclusive prefix;
                          // 0 (few blocks): the sweep adds the finished blocks itself
};

// Facts about where the grid's sizes fall among the samples, for batches whose
// tables share their sample sizes (the same for every table; written by
// k_batch_setup).  Intervals: 0 = below the first sample, i + 1 = from sample i on.
struct BatchPrep {
    double *rec;      // [n_m][BatchRec::slots]  everything about one message size (see BatchRec)
    double *tab;      // [2 + (n+1) + 2 n_s + 4 padded n_P]  interval of size 1 and 1 minus its start;
                      //                         widths of the intervals (the last: +inf); per candidate: s
                      //                         minus the start of its interval, then that interval; per
                      //                         process count: P - 1, floor(log2 P), ceil(log2 P) as
                      //                         doubles, then P - 1 and ceil(log2 P) as two uint32
};

// Entries of the per-process-count list of BatchPrep::tab: the grid's n_P, filled up to a
// multiple of eight, plus one.
__host__ __device__ inline long batch_padded_P(int n_P) { return ((long)n_P + 7) / 8 * 8 + 1; }

// Layout of one record of BatchPrep::rec, in 8-byte slots.
struct BatchRec {
    int DM;       // m minus the start of its interval
    int MD;       // m as a double
    int IM_NV;    // two int32: interval of m; candidates s <= min(m, s_cap)
    int D2;       // [cl_max] 2^j m minus the start of its interval
    int K;        // [n_s] k = ceil(m / s)
    int I2;       // [cl_max] int32: interval of 2^j m
    int JEND;     // [n+1] uint32: last j whose size j m lies in interval i
    int slots;
    __host__ __device__ BatchRec(int n, int n_s, int cl_max)
    {
        DM = 0; MD = 1; IM_NV = 2; D2 = 3;
        K = D2 + cl_max;
        I2 = K + n_s;
        JEND = I2 + (cl_max + 1) / 2;
        slots = JEND + (n + 2) / 2;
    }
};

// Per-(tables, grid) scratch in device memory, all written and read by kernels.
struct Scratch {
    double *g1;       // [n_tables]                       g(1)
    double *gs;       // [n_tables][n_s]                  g(s)
    double *gm;       // [n_tables][n_m]                  g(m)
    double *sum2;     // [n_tables][n_m][cl_max+1]        prefix over j of g(2^j m)
    double *blk;      // [n_tables][n_blk][n_m]           totals of the blocks of the chain sum
    double *pre;      // [n_tables][n_m][n_P]             sum of the blocks finished before each grid P (more than 32 blocks only)
    double *part;     // [n_tables][n_m][n_P]             in-block partial sums at the grid's P
    double *rcp;      // [n_s]                            1/s, rounded
    double *segC;     // [n_tables][n_s]                  C = g(s) + L
    double *segA;     // [n_tables][n_m][n_s]             A = g(s) ceil(m/s), +inf where s does not compete
    double *segB;     // [n_tables][n_m][n_s]             B = g(s) (ceil(m/s) - 1)   (both: n_s <= SWEEP_M_MAX_S only)
    double *amin;     // [n_tables][n_m]                  min over s of A (with segA, segB)
    int *nv;          // [n_m]                            candidates s <= min(m, s_cap)
    BatchPrep batch;  // shared sample sizes only
    double *batch_ys; // [n+2][n_tables][2]               {gap, slope} by interval (shared sample sizes only)
};

struct plogp_cell_dev {
    double time;
    uint32_t s;
    uint32_t strategy;
};

// What the kernels' launch shapes are sized by: read once from the device properties.
struct DeviceInfo {
    int n_cu;             // compute units
    size_t lds_per_cu;    // bytes of LDS of one compute unit
};
const DeviceInfo &device_info();

// Where each scratch array of a tune (or scoring) call starts inside one block of device
// memory, in bytes; every array starts on a 256-byte boundary.  An array the chosen path does
// not use has offset 0: the first 256 bytes of the block are a spare that nothing reads.
struct ScratchLayout {
    size_t g1, gs, gm, sum2, blk, pre, part, rcp, segC, segA, segB, amin, nv;
    size_t rec, tab, batch_ys;     // table-lane batch path
    size_t score_rows;             // scoring only: 2 doubles per (strategy, m)
    size_t total;                  // bytes of the block
};

enum TunePath : int { TUNE_TABLE_LANES = 0, TUNE_ROW = 1, TUNE_FUSED = 2, TUNE_STAGED = 3 };

// Everything the host decides about one tune call before the first launch: the path, every
// launch shape, and the scratch each kernel of that path reads or writes (one source for the
// allocation and for the kernels' index ranges).
struct TunePlan {
    int path;                      // TunePath
    int terms_only;                // the staged terms and sums only (scoring)
    ScratchLayout lay;
    // table-lane batch path
    int n_stage, prep_wg, n_tg, m_per_wave, batch_mchunks;
    size_t setup_lds, batch_lds;
    // whole-row path
    int row_two;
    size_t row_lds;
    // lane-per-m batch path
    int fused_mchunks;
    // staged path
    int lanes_s, lanes_p, pairs, terms_mode, n_chunks, n_mchunks, terms_wg;
    int chain, chain_row, together, row_together, terms_in_chain, chain_threads;
    int n_single, n_search, chain_wg, n_chain_wg, n_mgroups;
    size_t terms_lds, chain_lds, both_lds, crow_lds;
    int sweep_gp, sweep_ptiles;    // lanes over s
    int ppl, n_pg, n_w;            // lanes over P
    int n_mg, n_pcg;               // lanes over m
};

// Stages of a tune call, in launch order; a stage may launch nothing.
enum { TUNE_STAGE_TERMS = 0, TUNE_STAGE_CHAIN = 1, TUNE_STAGE_PREFIX = 2, TUNE_STAGE_SWEEP = 3,
       TUNE_STAGE_MORE = 4,       // the planes of the rows beyond Tables 1 and 2 (Gather, Barrier)
       TUNE_STAGES = 5 };

// Fills `plan`.  Returns false if a launch dimension or an index of the chosen path would not
// fit 31 bits (the job is too large for one call).
bool plan_tune(const DeviceTables &T, const DeviceGrid &G, bool terms_only, TunePlan &plan);
// The scratch arrays of a plan inside the block that starts at `base`.
Scratch bind_scratch(void *base, const ScratchLayout &lay);

// Each returns the hipError_t of the launch (hipGetLastError after it).
hipError_t launch_slopes(const DeviceTables &T, double *slope_out, hipStream_t st);
hipError_t launch_interp(const DeviceTables &T, int table, const uint64_t *d_z, size_t n,
                         double *d_out, hipStream_t st);
hipError_t launch_eval(const DeviceTables &T, int table, int strategy, const uint64_t *d_m,
                       const uint32_t *d_P, const uint64_t *d_s, size_t n, double *d_out,
                       hipStream_t st);
hipError_t launch_tune_stage(const TunePlan &plan, int stage, const DeviceTables &T, const DeviceGrid &G,
                             const Scratch &S, plogp_cell_dev *d_out, hipStream_t st);
inline hipError_t launch_tune(const TunePlan &plan, const DeviceTables &T, const DeviceGrid &G,
                              const Scratch &S, plogp_cell_dev *d_out, hipStream_t st)
{
    for (int stage = 0; stage < TUNE_STAGES; ++stage) {
        const hipError_t e = launch_tune_stage(plan, stage, T, G, S, d_out, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---- cut-over extraction (plogp_cutover.hip)
constexpr int CUT_TM = 16;                 // message sizes per thread (a tile of one row)
constexpr int CUT_SCAN_THREADS = 256;
constexpr int CUT_SCAN_PER = 8;            // counts per thread of the group scan
constexpr int CUT_SCAN_WG = CUT_SCAN_THREADS * CUT_SCAN_PER;

// Scratch of the cut-over extraction, one entry per (row, tile) unless noted.
struct CutScratch {
    uint32_t *counts;        // run starts in the tile
    uint32_t *local;         // their exclusive prefix inside a group of CUT_SCAN_WG entries
    uint32_t *flags;         // bit k: cell k of the tile starts a run
    uint64_t *group_total;   // [groups] totals, then their exclusive prefix
    uint64_t *ctl;           // one-pass path: [2 + workgroups] numbering, give-up flag, status words
};
constexpr int CUT_ROWS_KEEP = 8;           // run starts per row whose keys the one-pass path keeps in LDS
constexpr int CUT_ROWS_MAX_M = 512;        // sizes per row that the one-pass path keeps flags for
constexpr unsigned CUT_SPIN_LIMIT = 1u << 22;   // polls before a wait is given up (never reached)
// Whether the extraction takes the one-pass path, and the words of its control block.
bool cutover_by_rows(const DeviceGrid &G, int n_tables);
size_t cutover_ctl_words(const DeviceGrid &G, int n_tables);

// Number of (row, tile) entries for n_tables tables over grid G.
size_t cutover_items(const DeviceGrid &G, int n_tables);
// Stages: 0 mark the run starts, 1 prefix of their counts, 2 write the runs.
enum { CUT_STAGES = 3 };
hipError_t launch_cutovers_stage(int stage, const DeviceGrid &G, int n_tables, const plogp_cell_dev *d_cells,
                                 int key_mode, const CutScratch &C, uint64_t *d_row_offsets, void *d_runs,
                                 uint64_t capacity, hipStream_t st);

// Prediction against measurement for one table (T1: a view of that table alone).  plan: the
// terms-only plan of (T1, G), its scratch bound in S, score_rows among it.  Stages: 0 the
// terms and sums (the tune's own first stages), 1 predictions and verdicts, 2 statistics.
enum { SCORE_STAGES = 3 };
hipError_t launch_score_stage(int stage, const TunePlan &plan, const DeviceTables &T1, const DeviceGrid &G,
                              const Scratch &S, double *rows, const double *d_meas, const uint32_t *d_seg,
                              double *d_pred, void *d_verdict, void *d_scores, hipStream_t st);

// Robustness summary of n_tables decision tables of `cells` records each (table 0 is the
// reference).  d_max_dev and d_table_agree may be null.  cells < 2^40 and n_tables >= 1 are
// the caller's to check.
hipError_t launch_robustness(size_t cells, int n_tables, const plogp_cell_dev *d_cells, int key_mode,
                             uint32_t *d_agree, double *d_max_dev, uint32_t *d_table_agree,
                             hipStream_t st);

hipError_t kernels_init();

}  // namespace plogp
