// The opaque handles of the C ABI (include/plogp.h) and the host-side helpers that
// the entry points share.  Private to the library's own sources.
#pragma once

#include "../../include/plogp.h"
#include "plogp_internal.hpp"

namespace plogp {

// Records the HIP error for plogp_last_hip_error(), clears HIP's sticky error, returns PLOGP_EDEVICE.
int device_error(hipError_t e);
// One-time set-up of the library on the current device.
int ensure_init();

}  // namespace plogp

#define PLOGP_HIP_TRY(expr)                                     \
    do {                                                        \
        hipError_t e_ = (expr);                                 \
        if (e_ != hipSuccess) return plogp::device_error(e_);   \
    } while (0)

struct plogp_table {
    size_t n_tables = 0, n = 0;
    bool shared_x = false;      // every table has the sample sizes of the first one
    double *d_x = nullptr, *d_y = nullptr, *d_slope = nullptr, *d_L = nullptr;
    plogp::DeviceTables view() const
    {
        plogp::DeviceTables v;
        v.x = d_x; v.y = d_y; v.slope = d_slope; v.L = d_L;
        v.n = (int)n; v.n_tables = (int)n_tables;
        v.shared_x = shared_x ? 1 : 0;
        return v;
    }
    // the view of table `index` alone
    plogp::DeviceTables view_one(size_t index) const
    {
        plogp::DeviceTables v = view();
        v.x += index * n; v.y += index * n; v.slope += index * n; v.L += index;
        v.n_tables = 1;
        v.shared_x = 0;
        return v;
    }
    ~plogp_table();
};

struct plogp_grid {
    size_t n_m = 0, n_P = 0, n_s = 0;
    uint64_t s_cap = 0;
    uint32_t mask = 0;
    int n_ops = 0, n_blk = 0, last_terms = 0, cl_max = 0;
    uint64_t *d_m = nullptr, *d_s = nullptr, *d_mu = nullptr;
    uint32_t *d_P = nullptr;
    int *d_m_map = nullptr;
    size_t n_mu = 0;
    int *d_blk_off = nullptr;
    unsigned long long *d_blk_mask = nullptr;
    // scratch of the tuning and the scoring: one block, laid out per call by the call's plan
    void *scratch_block = nullptr;
    size_t scratch_bytes = 0;
    // scratch of the cut-over extraction, sized for cut_tables tables
    size_t cut_tables = 0;
    plogp::CutScratch cut = {};

    plogp::DeviceGrid view() const;
    void free_scratch();
    void free_cut_scratch();
    ~plogp_grid();
};

namespace plogp {

// Makes the grid's scratch block at least `bytes` long (waits for the device first if it has
// to be replaced: an earlier call on this handle may still run).
int ensure_scratch_block(plogp_grid *g, size_t bytes);
int ensure_cut_scratch(plogp_grid *g, size_t n_tables);

// Argument checks of the entry points, shared with their measured twins.
int check_tune_args(const plogp_table *t, const plogp_grid *g, const plogp_cell *d_out, size_t d_out_bytes);
int check_cutover_args(const plogp_grid *g, size_t n_tables, const plogp_cell *d_cells, int key_mode,
                       const uint64_t *d_row_offsets, const plogp_run *d_runs, size_t runs_capacity);
int check_score_args(const plogp_table *t, size_t table_index, const plogp_grid *g, const double *d_meas,
                     const uint32_t *d_seg, const double *d_pred, const plogp_verdict *d_verdict,
                     const plogp_strategy_score *d_scores);
int check_robust_args(const plogp_grid *g, size_t n_tables, const plogp_cell *d_cells, int key_mode,
                      const uint32_t *d_agree, const double *d_max_dev, const uint32_t *d_table_agree,
                      size_t *cells_out);

}  // namespace plogp
