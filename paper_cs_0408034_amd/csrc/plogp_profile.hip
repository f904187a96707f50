// Measurement twins of the C-ABI entry points (include/plogp_profile.h): the
// same per-stage launch functions as the product path, each stage launched
// `reps` times between two HIP events; and two kernels that measure what this
// device reaches on the fp64 vector and the HBM write roofline.  Nothing of the
// product path is in this file.
#include "../../include/plogp_profile.h"
#include "plogp_handles.hpp"

using namespace plogp;

#define HIP_TRY(expr) PLOGP_HIP_TRY(expr)

namespace {

// Runs stage(i) `reps` times between events i and i + 1, for i = 0..n_stages-1, waits, and
// writes the mean milliseconds per launch of every stage.
template <class Stage>
int timed_stages(int n_stages, int reps, hipStream_t st, float *ms_out, Stage stage)
{
    constexpr int MAX_STAGES = 5;
    hipEvent_t ev[MAX_STAGES + 1] = {};
    hipError_t e = hipSuccess;
    for (int i = 0; i <= n_stages && e == hipSuccess; ++i) e = hipEventCreate(&ev[i]);
    if (e == hipSuccess) e = hipEventRecord(ev[0], st);
    for (int i = 0; i < n_stages && e == hipSuccess; ++i) {
        for (int r = 0; r < reps && e == hipSuccess; ++r) e = stage(i);
        if (e == hipSuccess) e = hipEventRecord(ev[i + 1], st);
    }
    if (e == hipSuccess) e = hipEventSynchronize(ev[n_stages]);
    float ms[MAX_STAGES] = {0.f, 0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < n_stages && e == hipSuccess; ++i) {
        e = hipEventElapsedTime(&ms[i], ev[i], ev[i + 1]);
        ms[i] /= (float)reps;
    }
    for (int i = 0; i <= n_stages; ++i)
        if (ev[i]) (void)hipEventDestroy(ev[i]);
    if (e != hipSuccess) {
        // work may still be queued behind the failure: let it drain before the caller goes on
        (void)hipStreamSynchronize(st);
        return device_error(e);
    }
    for (int i = 0; i < n_stages; ++i) ms_out[i] = ms[i];
    return PLOGP_OK;
}

bool bad_reps(int reps) { return reps < 1 || reps > 10000; }

// ---- the two ceilings

constexpr int FMA_ACC = 8;

__global__ void __launch_bounds__(256) k_fma_peak(double *out, int iters, double a, double b)
{
    double v[FMA_ACC];
#pragma unroll
    for (int i = 0; i < FMA_ACC; ++i)
        v[i] = a + (double)threadIdx.x * 1e-9 + (double)i;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < FMA_ACC; ++i)
            v[i] = __builtin_fma(v[i], b, a);
    }
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < FMA_ACC; ++i)
        s = s + v[i];
    if (s == 12345.678)          // never true: keeps the arithmetic alive without a store per lane
        out[0] = s;
}

// STREAM: the stores carry the non-temporal hint, as the decision-table stores of the sweeps do.
template <bool STREAM>
__global__ void __launch_bounds__(256) k_store_fill(uint4 *buf, size_t n16, size_t per_wg)
{
    typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
    const size_t first = (size_t)blockIdx.x * per_wg;
    const size_t last = first + per_wg < n16 ? first + per_wg : n16;
    const u32x4_t v = {blockIdx.x, threadIdx.x, 0u, 0u};
    u32x4_t *out = reinterpret_cast<u32x4_t *>(buf);
    for (size_t i = first + threadIdx.x; i < last; i += 256) {
        if (STREAM)
            __builtin_nontemporal_store(v, out + i);
        else
            out[i] = v;
    }
}

}  // namespace

extern "C" {

int plogp_tune_grid_profile(const plogp_table *t, plogp_grid *g, plogp_cell *d_out,
                            size_t d_out_bytes, void *stream, int reps, float *stage_ms_out)
{
    if (!stage_ms_out || bad_reps(reps)) return PLOGP_EINVAL;
    int rc = check_tune_args(t, g, d_out, d_out_bytes);
    if (rc != PLOGP_OK) return rc;
    const DeviceTables T = t->view();
    const DeviceGrid G = g->view();
    TunePlan plan;
    if (!plan_tune(T, G, false, plan)) return PLOGP_ERANGE;
    if ((rc = ensure_scratch_block(g, plan.lay.total)) != PLOGP_OK) return rc;
    const Scratch S = bind_scratch(g->scratch_block, plan.lay);
    const hipStream_t st = (hipStream_t)stream;
    return timed_stages(TUNE_STAGES, reps, st, stage_ms_out, [&](int stage) {
        return launch_tune_stage(plan, stage, T, G, S, reinterpret_cast<plogp_cell_dev *>(d_out), st);
    });
}

int plogp_cutovers_profile(plogp_grid *g, size_t n_tables, const plogp_cell *d_cells, int key_mode,
                           uint64_t *d_row_offsets, plogp_run *d_runs, size_t runs_capacity,
                           void *stream, int reps, float *stage_ms_out)
{
    if (!stage_ms_out || bad_reps(reps)) return PLOGP_EINVAL;
    int rc = check_cutover_args(g, n_tables, d_cells, key_mode, d_row_offsets, d_runs, runs_capacity);
    if (rc != PLOGP_OK) return rc;
    if ((rc = ensure_init()) != PLOGP_OK) return rc;
    if ((rc = ensure_cut_scratch(g, n_tables)) != PLOGP_OK) return rc;
    const DeviceGrid G = g->view();
    const hipStream_t st = (hipStream_t)stream;
    return timed_stages(CUT_STAGES, reps, st, stage_ms_out, [&](int stage) {
        return launch_cutovers_stage(stage, G, (int)n_tables, reinterpret_cast<const plogp_cell_dev *>(d_cells),
                                     key_mode, g->cut, d_row_offsets, d_runs, runs_capacity, st);
    });
}

int plogp_score_grid_profile(const plogp_table *t, size_t table_index, plogp_grid *g,
                             const double *d_meas, const uint32_t *d_seg, double *d_pred,
                             plogp_verdict *d_verdict, plogp_strategy_score *d_scores, void *stream,
                             int reps, float *stage_ms_out)
{
    if (!stage_ms_out || bad_reps(reps)) return PLOGP_EINVAL;
    int rc = check_score_args(t, table_index, g, d_meas, d_seg, d_pred, d_verdict, d_scores);
    if (rc != PLOGP_OK) return rc;
    if ((rc = ensure_init()) != PLOGP_OK) return rc;
    const DeviceTables T1 = t->view_one(table_index);
    const DeviceGrid G = g->view();
    TunePlan plan;
    if (!plan_tune(T1, G, true, plan)) return PLOGP_ERANGE;
    if ((rc = ensure_scratch_block(g, plan.lay.total)) != PLOGP_OK) return rc;
    const Scratch S = bind_scratch(g->scratch_block, plan.lay);
    double *rows = reinterpret_cast<double *>(static_cast<char *>(g->scratch_block) + plan.lay.score_rows);
    const hipStream_t st = (hipStream_t)stream;
    return timed_stages(SCORE_STAGES, reps, st, stage_ms_out, [&](int stage) {
        return launch_score_stage(stage, plan, T1, G, S, rows, d_meas, d_seg, d_pred, d_verdict, d_scores, st);
    });
}

int plogp_robustness_profile(const plogp_grid *g, size_t n_tables, const plogp_cell *d_cells,
                             int key_mode, uint32_t *d_agree, double *d_max_dev,
                             uint32_t *d_table_agree, void *stream, int reps, float *ms_out)
{
    if (!ms_out || bad_reps(reps)) return PLOGP_EINVAL;
    size_t cells = 0;
    int rc = check_robust_args(g, n_tables, d_cells, key_mode, d_agree, d_max_dev, d_table_agree, &cells);
    if (rc != PLOGP_OK) return rc;
    if ((rc = ensure_init()) != PLOGP_OK) return rc;
    const hipStream_t st = (hipStream_t)stream;
    return timed_stages(1, reps, st, ms_out, [&](int) {
        return launch_robustness(cells, (int)n_tables, reinterpret_cast<const plogp_cell_dev *>(d_cells),
                                 key_mode, d_agree, d_max_dev, d_table_agree, st);
    });
}

int plogp_measure_ceilings(void *d_buf, size_t buf_bytes, void *stream, double *fma_tflops_out,
                           double *store_gbs_out)
{
    if (!d_buf || !fma_tflops_out || !store_gbs_out || buf_bytes < 16 || ((uintptr_t)d_buf & 15u) != 0)
        return PLOGP_EINVAL;
    int rc = ensure_init();
    if (rc != PLOGP_OK) return rc;
    const hipStream_t st = (hipStream_t)stream;
    const int n_cu = device_info().n_cu;
    // fp64 multiply-adds: 8 workgroups of 4 waves per compute unit = 8 waves per SIMD
    const int fma_blocks = n_cu * 8, fma_iters = 4096;
    const double fma_flops = (double)fma_blocks * 256.0 * fma_iters * FMA_ACC * 2.0;
    // the fill: 16 workgroups per compute unit, each a contiguous slice
    const size_t n16 = buf_bytes / 16;
    const size_t fill_blocks = (size_t)n_cu * 16;
    const size_t per_wg = (n16 + fill_blocks - 1) / fill_blocks;
    float best[3] = {0.f, 0.f, 0.f};                    // multiply-adds, plain fill, streaming fill
    for (int which = 0; which < 3; ++which) {
        for (int round = 0; round < 4; ++round) {       // round 0 warms up
            float ms = 0.f;
            rc = timed_stages(1, 1, st, &ms, [&](int) {
                if (which == 0)
                    hipLaunchKernelGGL(k_fma_peak, dim3(fma_blocks), dim3(256), 0, st,
                                       static_cast<double *>(d_buf), fma_iters, 1.0, 1.0000001);
                else
                    hipLaunchKernelGGL(which == 1 ? k_store_fill<false> : k_store_fill<true>,
                                       dim3((unsigned)fill_blocks), dim3(256), 0, st,
                                       static_cast<uint4 *>(d_buf), n16, per_wg);
                return hipGetLastError();
            });
            if (rc != PLOGP_OK) return rc;
            if (round > 0 && (best[which] == 0.f || ms < best[which])) best[which] = ms;
        }
    }
    *fma_tflops_out = fma_flops / ((double)best[0] * 1e-3) / 1e12;
    const float fill_ms = best[2] < best[1] ? best[2] : best[1];
    *store_gbs_out = (double)(n16 * 16) / ((double)fill_ms * 1e-3) / 1e9;
    return PLOGP_OK;
}

}  // extern "C"
