/*
 * plogp_profile.h -- measurement interface of libplogp (benchmarks only).
 *
 * Not part of the product path: these entry points do the same work as their
 * twins in plogp.h through the same per-stage launch functions, but launch
 * every stage `reps` times back to back between two HIP events on `stream`
 * (each launch rewrites the same outputs with the same values), wait for
 * completion and return the mean milliseconds per launch of each stage.  A
 * single pair of events around a 10 us kernel would mostly measure the launch
 * gap; `reps` launches between the events measure the kernel.
 *
 * All are synchronous.  Errors: as the twin, plus PLOGP_EINVAL for a null
 * output pointer or reps outside [1, 10000].
 */
#ifndef PLOGP_PROFILE_H
#define PLOGP_PROFILE_H

#include "plogp.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Twin of plogp_tune_grid (paper Section 3.1 / Section 1: the sweep).
 * stage_ms_out[0..4]:
 *   [0] per-table and per-m terms (interval slopes, g(1), g(s), g(m), the
 *       Scatter-binomial prefix sums), [1] Scatter-chain block sums,
 *   [2] Scatter-chain block prefix, [3] sweep + arg-min + decision-table write,
 *   [4] the planes of the rows beyond Tables 1 and 2 (Gather, Barrier), if enabled.
 * A stage that launched nothing reports 0.  For tables of up to about 1000
 * samples the terms and the Scatter-chain block sums are one launch, reported
 * under [1]; the paths that do everything in one kernel (batches of tables; one
 * workgroup per (table, m) row) report it under [3].
 */
int plogp_tune_grid_profile(const plogp_table *t, plogp_grid *g, plogp_cell *d_out,
                            size_t d_out_bytes, void *stream, int reps, float *stage_ms_out);

/* Twin of plogp_cutovers.  stage_ms_out[0..2]: mark run starts, prefix of their
 * counts, write the runs. */
int plogp_cutovers_profile(plogp_grid *g, size_t n_tables, const plogp_cell *d_cells, int key_mode,
                           uint64_t *d_row_offsets, plogp_run *d_runs, size_t runs_capacity,
                           void *stream, int reps, float *stage_ms_out);

/* Twin of plogp_score_grid.  stage_ms_out[0..2]: g(m), g(1) and the Scatter
 * sums; predictions and verdicts; statistics. */
int plogp_score_grid_profile(const plogp_table *t, size_t table_index, plogp_grid *g,
                             const double *d_meas, const uint32_t *d_seg, double *d_pred,
                             plogp_verdict *d_verdict, plogp_strategy_score *d_scores, void *stream,
                             int reps, float *stage_ms_out);

/* Twin of plogp_robustness.  *ms_out: clearing the outputs included. */
int plogp_robustness_profile(const plogp_grid *g, size_t n_tables, const plogp_cell *d_cells,
                             int key_mode, uint32_t *d_agree, double *d_max_dev,
                             uint32_t *d_table_agree, void *stream, int reps, float *ms_out);

/*
 * What this device reaches on the two rooflines the sweep is priced against,
 * measured here and now, to be quoted beside the published peaks:
 *   *fma_tflops_out    fp64 vector rate of a kernel that does nothing but
 *                      independent fused multiply-adds (8 waves per SIMD, eight
 *                      accumulators per lane), in TFLOP/s (a multiply-add = 2);
 *   *store_gbs_out     write bandwidth of a kernel that does nothing but fill
 *                      d_buf (DEVICE, at least 16 bytes, 16-byte aligned; its
 *                      contents are overwritten) with 16-byte stores, a wave
 *                      writing 1 KB runs, in GB/s: the faster of a fill with
 *                      plain stores and one with non-temporal stores.
 * Each is the best of three launches after a warm-up launch.  Synchronous.
 * Errors: EINVAL (null, misaligned, buf_bytes < 16), EDEVICE.
 */
int plogp_measure_ceilings(void *d_buf, size_t buf_bytes, void *stream, double *fma_tflops_out,
                           double *store_gbs_out);

#ifdef __cplusplus
}
#endif
#endif /* PLOGP_PROFILE_H */
