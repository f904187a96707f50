// C ABI of the pLogP tuning library (see include/plogp.h): handle management,
// argument validation and stream plumbing.  All arithmetic of the method is
// in plogp_kernels.hip; nothing here evaluates a model or interpolates g().
#include "../../include/plogp.h"
#include "plogp_internal.hpp"

#include <algorithm>
#include <math.h>
#include <mutex>
#include <new>
#include <vector>

using namespace plogp;

namespace {

thread_local int tl_hip_error = 0;

int device_error(hipError_t e)
{
    tl_hip_error = (int)e;
    (void)hipGetLastError();   // clear the sticky error so the next call starts clean
    return PLOGP_EDEVICE;
}

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) return device_error(e_);  \
    } while (0)

constexpr double kTwo53 = 9007199254740992.0;
constexpr uint64_t kTwo53u = 1ull << 53;

bool g_init_done = false;
std::mutex g_init_mutex;

int ensure_init()
{
    std::lock_guard<std::mutex> lock(g_init_mutex);
    if (!g_init_done) {
        int count = 0;
        HIP_TRY(hipGetDeviceCount(&count));
        if (count < 1) return device_error(hipErrorNoDevice);
        HIP_TRY(kernels_init());
        g_init_done = true;
    }
    return PLOGP_OK;
}

int floor_log2_u32(uint32_t v) { int f = 0; while ((v >> (f + 1)) != 0) ++f; return f; }
int ceil_log2_u32(uint32_t v) { int f = floor_log2_u32(v); return ((1u << f) == v) ? f : f + 1; }

}  // namespace

struct plogp_table {
    size_t n_tables = 0, n = 0;
    bool shared_x = false;      // every table has the sample sizes of the first one
    double *d_x = nullptr, *d_y = nullptr, *d_slope = nullptr, *d_L = nullptr;
    DeviceTables view() const
    {
        DeviceTables v;
        v.x = d_x; v.y = d_y; v.slope = d_slope; v.L = d_L;
        v.n = (int)n; v.n_tables = (int)n_tables;
        v.shared_x = shared_x ? 1 : 0;
        return v;
    }
    ~plogp_table()
    {
        if (d_x) (void)hipFree(d_x);
        if (d_y) (void)hipFree(d_y);
        if (d_slope) (void)hipFree(d_slope);
        if (d_L) (void)hipFree(d_L);
    }
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
    // scratch, sized for scratch_tables tables
    size_t scratch_tables = 0, scratch_samples = 0;
    Scratch scratch = {};
    // scratch of the path for batches with shared sample sizes
    size_t batch_tables = 0, batch_samples = 0;
    // scratch of the scoring: 2 doubles per (strategy, m)
    double *score_rows = nullptr;
    // scratch of the cut-over extraction, sized for cut_tables tables
    size_t cut_tables = 0;
    CutScratch cut = {};

    DeviceGrid view() const
    {
        DeviceGrid g;
        g.m = d_m; g.P = d_P; g.s = d_s; g.blk_off = d_blk_off; g.blk_mask = d_blk_mask;
        g.mu = d_mu; g.m_map = d_m_map; g.n_mu = (int)n_mu;
        g.n_m = (int)n_m; g.n_P = (int)n_P; g.n_s = (int)n_s;
        g.n_blk = n_blk; g.last_terms = last_terms; g.cl_max = cl_max;
        g.s_cap = s_cap; g.mask = mask; g.n_ops = n_ops;
        g.blk_is_prefix = n_blk > 32 ? 1 : 0;
        return g;
    }
    void free_scratch()
    {
        double **all[] = {&scratch.g1, &scratch.gs, &scratch.gm, &scratch.sum2, &scratch.blk,
                          &scratch.pre, &scratch.part, &scratch.rcp,
                          &scratch.segC, &scratch.segA, &scratch.segB, &scratch.amin};
        for (double **p : all) {
            if (*p) (void)hipFree(*p);
            *p = nullptr;
        }
        if (scratch.nv) (void)hipFree(scratch.nv);
        scratch.nv = nullptr;
        scratch_tables = 0;
        scratch_samples = 0;
    }
    void free_batch_scratch()
    {
        BatchPrep &b = scratch.batch;
        void *all[] = {b.rec, b.tab, scratch.batch_ys};
        for (void *p : all)
            if (p) (void)hipFree(p);
        b = BatchPrep{};
        scratch.batch_ys = nullptr;
        batch_tables = batch_samples = 0;
    }
    void free_cut_scratch()
    {
        if (cut.counts) (void)hipFree(cut.counts);
        if (cut.local) (void)hipFree(cut.local);
        if (cut.flags) (void)hipFree(cut.flags);
        if (cut.group_total) (void)hipFree(cut.group_total);
        cut = CutScratch{};
        cut_tables = 0;
    }
    ~plogp_grid()
    {
        free_scratch();
        free_batch_scratch();
        free_cut_scratch();
        if (score_rows) (void)hipFree(score_rows);
        if (d_m) (void)hipFree(d_m);
        if (d_mu) (void)hipFree(d_mu);
        if (d_m_map) (void)hipFree(d_m_map);
        if (d_s) (void)hipFree(d_s);
        if (d_P) (void)hipFree(d_P);
        if (d_blk_off) (void)hipFree(d_blk_off);
        if (d_blk_mask) (void)hipFree(d_blk_mask);
    }
};

extern "C" {

const char *plogp_strerror(int status)
{
    switch (status) {
    case PLOGP_OK: return "ok";
    case PLOGP_EINVAL: return "invalid argument";
    case PLOGP_ERANGE: return "a size entering a model would reach 2^53";
    case PLOGP_ENOSPC: return "output buffer too small";
    case PLOGP_ENOMEM: return "out of memory";
    case PLOGP_EDEVICE: return "HIP error (see plogp_last_hip_error)";
    default: return "unknown status";
    }
}

int plogp_last_hip_error(void) { return tl_hip_error; }

int plogp_load_tables(const double *sizes, const double *gaps, size_t n, const double *L,
                      size_t n_tables, plogp_table **out)
{
    if (!sizes || !gaps || !L || !out) return PLOGP_EINVAL;
    if (n < 2 || n > PLOGP_MAX_SAMPLES || n_tables < 1 || n_tables > (1u << 24)) return PLOGP_EINVAL;
    for (size_t t = 0; t < n_tables; ++t) {
        if (!(L[t] >= 0.0 && L[t] <= PLOGP_MAX_TIME)) return PLOGP_EINVAL;
        const double *x = sizes + t * n, *y = gaps + t * n;
        for (size_t i = 0; i < n; ++i) {
            if (!(x[i] >= 1.0 && x[i] < kTwo53) || x[i] != floor(x[i])) return PLOGP_EINVAL;
            if (i > 0 && !(x[i] > x[i - 1])) return PLOGP_EINVAL;
            if (!(y[i] >= 0.0 && y[i] <= PLOGP_MAX_TIME)) return PLOGP_EINVAL;
        }
    }
    int rc = ensure_init();
    if (rc != PLOGP_OK) return rc;
    plogp_table *h = new (std::nothrow) plogp_table;
    if (!h) return PLOGP_ENOMEM;
    h->n = n;
    h->n_tables = n_tables;
    h->shared_x = true;
    for (size_t t = 1; t < n_tables && h->shared_x; ++t)
        for (size_t i = 0; i < n; ++i)
            if (sizes[t * n + i] != sizes[i]) { h->shared_x = false; break; }
    const size_t bytes = n_tables * n * sizeof(double);
    hipError_t e;
    if ((e = hipMalloc((void **)&h->d_x, bytes)) != hipSuccess ||
        (e = hipMalloc((void **)&h->d_y, bytes)) != hipSuccess ||
        (e = hipMalloc((void **)&h->d_slope, bytes)) != hipSuccess ||
        (e = hipMalloc((void **)&h->d_L, n_tables * sizeof(double))) != hipSuccess) {
        delete h;
        if (e == hipErrorOutOfMemory) { (void)hipGetLastError(); return PLOGP_ENOMEM; }
        return device_error(e);
    }
    if ((e = hipMemcpy(h->d_x, sizes, bytes, hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(h->d_y, gaps, bytes, hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(h->d_L, L, n_tables * sizeof(double), hipMemcpyHostToDevice)) != hipSuccess ||
        (e = launch_slopes(h->view(), nullptr)) != hipSuccess ||
        (e = hipStreamSynchronize(nullptr)) != hipSuccess) {
        delete h;
        return device_error(e);
    }
    *out = h;
    return PLOGP_OK;
}

int plogp_load_table(const double *sizes, const double *gaps, size_t n, double L, plogp_table **out)
{
    return plogp_load_tables(sizes, gaps, n, &L, 1, out);
}

int plogp_free_table(plogp_table *t)
{
    delete t;
    return PLOGP_OK;
}

size_t plogp_table_count(const plogp_table *t) { return t ? t->n_tables : 0; }
size_t plogp_table_samples(const plogp_table *t) { return t ? t->n : 0; }

int plogp_table_slopes(const plogp_table *t, size_t table_index, double *slopes_out, size_t n)
{
    if (!t || !slopes_out || table_index >= t->n_tables || n != t->n) return PLOGP_EINVAL;
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(slopes_out, t->d_slope + table_index * t->n, n * sizeof(double),
                      hipMemcpyDeviceToHost));
    return PLOGP_OK;
}

int plogp_interp_g(const plogp_table *t, size_t table_index, const uint64_t *d_z, size_t n,
                   double *d_g_out, void *stream)
{
    if (!t || table_index >= t->n_tables) return PLOGP_EINVAL;
    if (n == 0) return PLOGP_OK;
    if (!d_z || !d_g_out) return PLOGP_EINVAL;
    HIP_TRY(launch_interp(t->view(), (int)table_index, d_z, n, d_g_out, (hipStream_t)stream));
    return PLOGP_OK;
}

int plogp_eval_strategy(const plogp_table *t, size_t table_index, int strategy, const uint64_t *d_m,
                        const uint32_t *d_P, const uint64_t *d_s, size_t n, double *d_time_out,
                        void *stream)
{
    if (!t || table_index >= t->n_tables) return PLOGP_EINVAL;
    if (strategy < 0 || strategy >= PLOGP_N_STRATEGIES) return PLOGP_EINVAL;
    if (n == 0) return PLOGP_OK;
    const bool seg = strategy == 2 || strategy == 5 || strategy == 9;
    if (!d_m || !d_P || !d_time_out || (seg && !d_s)) return PLOGP_EINVAL;
    HIP_TRY(launch_eval(t->view(), (int)table_index, strategy, d_m, d_P, d_s, n, d_time_out,
                        (hipStream_t)stream));
    return PLOGP_OK;
}

int plogp_grid_create(const plogp_grid_desc *d, plogp_grid **out)
{
    if (!d || !out) return PLOGP_EINVAL;
    if (d->n_m == 0 || d->n_P == 0 || !d->m || !d->P) return PLOGP_EINVAL;
    if (d->n_s > 0 && !d->s) return PLOGP_EINVAL;
    if (d->n_m > (1u << 24) || d->n_P > (1u << 24) || d->n_s > (1u << 24)) return PLOGP_EINVAL;
    const uint32_t mask = d->strategy_mask & PLOGP_MASK_ALL;
    if (mask == 0 || mask != d->strategy_mask) return PLOGP_EINVAL;
    const uint64_t unit = d->dtype_size > 1 ? d->dtype_size : 1;
    uint64_t m_max = 0;
    bool too_big = false;
    for (size_t i = 0; i < d->n_m; ++i) {
        if (d->m[i] == 0 || d->m[i] % unit != 0) return PLOGP_EINVAL;
        if (d->m[i] >= kTwo53u) too_big = true;
        if (d->m[i] > m_max) m_max = d->m[i];
    }
    for (size_t i = 0; i < d->n_P; ++i) {
        if (d->P[i] < 2) return PLOGP_EINVAL;
        if (i > 0 && d->P[i] <= d->P[i - 1]) return PLOGP_EINVAL;
    }
    for (size_t i = 0; i < d->n_s; ++i) {
        if (d->s[i] == 0 || d->s[i] >= (1ull << 32) || d->s[i] % unit != 0) return PLOGP_EINVAL;
        if (i > 0 && d->s[i] <= d->s[i - 1]) return PLOGP_EINVAL;
    }
    if (too_big) return PLOGP_ERANGE;
    const uint32_t Pmax = d->P[d->n_P - 1];
    const int cl_max = ceil_log2_u32(Pmax);
    if ((mask & (1u << 11)) && (uint64_t)(Pmax - 1) > (kTwo53u - 1) / m_max) return PLOGP_ERANGE;
    if ((mask & (1u << 12)) && m_max > ((kTwo53u - 1) >> (cl_max > 0 ? cl_max - 1 : 0)))
        return PLOGP_ERANGE;

    int rc = ensure_init();
    if (rc != PLOGP_OK) return rc;

    plogp_grid *g = new (std::nothrow) plogp_grid;
    if (!g) return PLOGP_ENOMEM;
    g->n_m = d->n_m; g->n_P = d->n_P; g->n_s = d->n_s;
    g->s_cap = d->s_cap;
    g->mask = mask;
    g->n_ops = ((mask & PLOGP_MASK_BCAST) ? 1 : 0) + ((mask & PLOGP_MASK_SCATTER) ? 1 : 0);
    g->cl_max = cl_max;
    g->n_blk = (int)((Pmax - 1) / SUM_BLOCK) + 1;
    g->last_terms = (int)((Pmax - 1) - (uint32_t)SUM_BLOCK * (uint32_t)(g->n_blk - 1));
    // P indices per block of the Scatter-chain sum: block b holds the P with (P-1)/SUM_BLOCK == b
    std::vector<int> off((size_t)g->n_blk + 1, 0);
    std::vector<unsigned long long> bmask((size_t)g->n_blk, 0ull);
    static_assert(SUM_BLOCK == 64, "one 64-bit mask per block");
    for (size_t i = 0; i < d->n_P; ++i) {
        off[(d->P[i] - 1) / SUM_BLOCK + 1] += 1;
        bmask[(d->P[i] - 1) / SUM_BLOCK] |= 1ull << ((d->P[i] - 1) % SUM_BLOCK);
    }
    for (int b = 0; b < g->n_blk; ++b) off[b + 1] += off[b];
    // the distinct message sizes (index metadata: grids of log-spaced sizes rounded to the
    // datatype repeat small sizes, and equal sizes have equal Scatter-chain sums)
    std::vector<uint64_t> mu(d->m, d->m + d->n_m);
    std::sort(mu.begin(), mu.end());
    mu.erase(std::unique(mu.begin(), mu.end()), mu.end());
    std::vector<int> m_map(d->n_m);
    for (size_t i = 0; i < d->n_m; ++i)
        m_map[i] = (int)(std::lower_bound(mu.begin(), mu.end(), d->m[i]) - mu.begin());
    g->n_mu = mu.size();

    hipError_t e;
    if ((e = hipMalloc((void **)&g->d_m, d->n_m * sizeof(uint64_t))) != hipSuccess ||
        (e = hipMalloc((void **)&g->d_mu, mu.size() * sizeof(uint64_t))) != hipSuccess ||
        (e = hipMalloc((void **)&g->d_m_map, d->n_m * sizeof(int))) != hipSuccess ||
        (e = hipMalloc((void **)&g->d_P, d->n_P * sizeof(uint32_t))) != hipSuccess ||
        (e = hipMalloc((void **)&g->d_s, (d->n_s ? d->n_s : 1) * sizeof(uint64_t))) != hipSuccess ||
        (e = hipMalloc((void **)&g->d_blk_off, off.size() * sizeof(int))) != hipSuccess ||
        (e = hipMalloc((void **)&g->d_blk_mask, bmask.size() * sizeof(unsigned long long))) != hipSuccess) {
        delete g;
        if (e == hipErrorOutOfMemory) { (void)hipGetLastError(); return PLOGP_ENOMEM; }
        return device_error(e);
    }
    if ((e = hipMemcpy(g->d_m, d->m, d->n_m * sizeof(uint64_t), hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(g->d_mu, mu.data(), mu.size() * sizeof(uint64_t), hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(g->d_m_map, m_map.data(), d->n_m * sizeof(int), hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(g->d_P, d->P, d->n_P * sizeof(uint32_t), hipMemcpyHostToDevice)) != hipSuccess ||
        (d->n_s && (e = hipMemcpy(g->d_s, d->s, d->n_s * sizeof(uint64_t), hipMemcpyHostToDevice)) != hipSuccess) ||
        (e = hipMemcpy(g->d_blk_off, off.data(), off.size() * sizeof(int), hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(g->d_blk_mask, bmask.data(), bmask.size() * sizeof(unsigned long long), hipMemcpyHostToDevice)) != hipSuccess) {
        delete g;
        return device_error(e);
    }
    *out = g;
    return PLOGP_OK;
}

int plogp_grid_free(plogp_grid *g)
{
    delete g;
    return PLOGP_OK;
}

size_t plogp_grid_ops(const plogp_grid *g) { return g ? (size_t)g->n_ops : 0; }

size_t plogp_decision_table_cells(size_t n_tables, const plogp_grid *g)
{
    return g ? n_tables * (size_t)g->n_ops * g->n_m * g->n_P : 0;
}

size_t plogp_decision_table_bytes(size_t n_tables, const plogp_grid *g)
{
    return plogp_decision_table_cells(n_tables, g) * sizeof(plogp_cell);
}

static int ensure_scratch(plogp_grid *g, size_t n_tables, size_t n_samples)
{
    if (g->scratch_tables >= n_tables && g->scratch_samples >= n_samples) return PLOGP_OK;
    // a previous tune on this handle may still be running on some stream
    HIP_TRY(hipDeviceSynchronize());
    g->free_scratch();
    const bool chain = (g->mask & (1u << 11)) != 0, binom = (g->mask & (1u << 12)) != 0;
    const bool pairs = g->n_s > 0 && g->n_s <= (size_t)SWEEP_M_MAX_S && g->n_P >= 32;
    struct { double **p; size_t count; } want[] = {
        {&g->scratch.g1, n_tables},
        {&g->scratch.gs, n_tables * (g->n_s ? g->n_s : 1)},
        {&g->scratch.gm, n_tables * g->n_m},
        {&g->scratch.sum2, binom ? n_tables * g->n_m * (size_t)(g->cl_max + 1) : 1},
        {&g->scratch.blk, chain ? n_tables * (size_t)g->n_blk * g->n_m : 1},
        {&g->scratch.part, chain ? n_tables * g->n_m * g->n_P : 1},
        {&g->scratch.rcp, g->n_s ? g->n_s : 1},
        {&g->scratch.pre, chain && g->n_blk > 32 ? n_tables * g->n_m * g->n_P : 1},
        {&g->scratch.segC, n_tables * (g->n_s ? g->n_s : 1)},
        {&g->scratch.segA, pairs ? n_tables * g->n_m * g->n_s : 1},
        {&g->scratch.segB, pairs ? n_tables * g->n_m * g->n_s : 1},
        {&g->scratch.amin, pairs ? n_tables * g->n_m : 1},
    };
    for (auto &w : want) {
        hipError_t e = hipMalloc((void **)w.p, w.count * sizeof(double));
        if (e != hipSuccess) {
            g->free_scratch();
            if (e == hipErrorOutOfMemory) { (void)hipGetLastError(); return PLOGP_ENOMEM; }
            return device_error(e);
        }
    }
    {
        hipError_t e = hipMalloc((void **)&g->scratch.nv, g->n_m * sizeof(int));
        if (e != hipSuccess) {
            g->free_scratch();
            if (e == hipErrorOutOfMemory) { (void)hipGetLastError(); return PLOGP_ENOMEM; }
            return device_error(e);
        }
    }
    g->scratch_tables = n_tables;
    g->scratch_samples = n_samples;
    return PLOGP_OK;
}

static int ensure_batch_scratch(plogp_grid *g, size_t n_tables, size_t n)
{
    if (g->batch_tables >= n_tables && g->batch_samples == n) return PLOGP_OK;
    HIP_TRY(hipDeviceSynchronize());     // an earlier tune on this handle may still run
    g->free_batch_scratch();
    BatchPrep &b = g->scratch.batch;
    const BatchRec R((int)n, (int)g->n_s, g->cl_max);
    struct { void **p; size_t bytes; } want[] = {
        {(void **)&b.rec, g->n_m * (size_t)R.slots * sizeof(double)},
        {(void **)&b.tab, (2 + (n + 1) + 2 * (g->n_s ? g->n_s : 1) + 3 * g->n_P) * sizeof(double)},
        {(void **)&g->scratch.batch_ys, (n + 2) * n_tables * 2 * sizeof(double)},
    };
    for (auto &w : want) {
        hipError_t e = hipMalloc(w.p, w.bytes);
        if (e != hipSuccess) {
            g->free_batch_scratch();
            if (e == hipErrorOutOfMemory) { (void)hipGetLastError(); return PLOGP_ENOMEM; }
            return device_error(e);
        }
    }
    g->batch_tables = n_tables;
    g->batch_samples = n;
    return PLOGP_OK;
}

// Scratch for whichever path launch_tune will take.
static int ensure_tune_scratch(const plogp_table *t, plogp_grid *g)
{
    if (use_table_lane_path(t->view(), g->view())) return ensure_batch_scratch(g, t->n_tables, t->n);
    if (use_fused_path(t->view(), g->view()) || use_row_path(t->view(), g->view())) return PLOGP_OK;
    return ensure_scratch(g, t->n_tables, t->n);
}

int plogp_tune_grid(const plogp_table *t, plogp_grid *g, plogp_cell *d_out, size_t d_out_bytes,
                    void *stream)
{
    if (!t || !g || !d_out) return PLOGP_EINVAL;
    if (((uintptr_t)d_out & 15u) != 0) return PLOGP_EINVAL;
    if (d_out_bytes < plogp_decision_table_bytes(t->n_tables, g)) return PLOGP_ENOSPC;
    {
        int rc = ensure_tune_scratch(t, g);
        if (rc != PLOGP_OK) return rc;
    }
    HIP_TRY(launch_tune(t->view(), g->view(), g->scratch,
                        reinterpret_cast<plogp_cell_dev *>(d_out), (hipStream_t)stream));
    return PLOGP_OK;
}

int plogp_tune_grid_profile(const plogp_table *t, plogp_grid *g, plogp_cell *d_out,
                            size_t d_out_bytes, void *stream, int reps, float *stage_ms_out)
{
    if (!t || !g || !d_out || !stage_ms_out || reps < 1 || reps > 10000) return PLOGP_EINVAL;
    if (((uintptr_t)d_out & 15u) != 0) return PLOGP_EINVAL;
    if (d_out_bytes < plogp_decision_table_bytes(t->n_tables, g)) return PLOGP_ENOSPC;
    {
        int rc = ensure_tune_scratch(t, g);
        if (rc != PLOGP_OK) return rc;
    }
    hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
    hipError_t e = hipSuccess;
    for (int i = 0; i < 5 && e == hipSuccess; ++i) e = hipEventCreate(&ev[i]);
    if (e == hipSuccess)
        e = launch_tune(t->view(), g->view(), g->scratch, reinterpret_cast<plogp_cell_dev *>(d_out),
                        (hipStream_t)stream, ev, reps);
    if (e == hipSuccess) e = hipEventSynchronize(ev[4]);
    float ms[4] = {0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < 4 && e == hipSuccess; ++i) {
        e = hipEventElapsedTime(&ms[i], ev[i], ev[i + 1]);
        ms[i] /= (float)reps;
    }
    for (int i = 0; i < 5; ++i)
        if (ev[i]) (void)hipEventDestroy(ev[i]);
    if (e != hipSuccess) return device_error(e);
    const bool table_lanes = use_table_lane_path(t->view(), g->view());
    const bool fused = table_lanes || use_fused_path(t->view(), g->view()) || use_row_path(t->view(), g->view());
    const bool chain = (g->mask & (1u << 11)) != 0 && !fused;
    if (fused && !table_lanes) ms[0] = 0.f;
    stage_ms_out[0] = ms[0];
    stage_ms_out[1] = chain ? ms[1] : 0.f;
    stage_ms_out[2] = chain ? ms[2] : 0.f;
    stage_ms_out[3] = ms[3];
    return PLOGP_OK;
}

static int ensure_cut_scratch(plogp_grid *g, size_t n_tables)
{
    if (g->cut_tables >= n_tables) return PLOGP_OK;
    HIP_TRY(hipDeviceSynchronize());     // an earlier extraction on this handle may still run
    g->free_cut_scratch();
    const size_t items = cutover_items(g->view(), (int)n_tables);
    const size_t groups = (items + CUT_SCAN_WG - 1) / CUT_SCAN_WG;
    hipError_t e;
    if ((e = hipMalloc((void **)&g->cut.counts, items * sizeof(uint32_t))) != hipSuccess ||
        (e = hipMalloc((void **)&g->cut.local, items * sizeof(uint32_t))) != hipSuccess ||
        (e = hipMalloc((void **)&g->cut.flags, items * sizeof(uint32_t))) != hipSuccess ||
        (e = hipMalloc((void **)&g->cut.group_total, (groups ? groups : 1) * sizeof(uint64_t))) != hipSuccess) {
        g->free_cut_scratch();
        if (e == hipErrorOutOfMemory) { (void)hipGetLastError(); return PLOGP_ENOMEM; }
        return device_error(e);
    }
    g->cut_tables = n_tables;
    return PLOGP_OK;
}

static int check_cutover_args(const plogp_grid *g, size_t n_tables, const plogp_cell *d_cells,
                              int key_mode, const uint64_t *d_row_offsets, const plogp_run *d_runs,
                              size_t runs_capacity)
{
    if (!g || !d_cells || !d_row_offsets || n_tables < 1 || n_tables > (1u << 24)) return PLOGP_EINVAL;
    if (key_mode != PLOGP_KEY_STRATEGY && key_mode != PLOGP_KEY_STRATEGY_AND_SEGMENT) return PLOGP_EINVAL;
    if (runs_capacity > 0 && !d_runs) return PLOGP_EINVAL;
    if (((uintptr_t)d_cells & 15u) != 0 || ((uintptr_t)d_runs & 15u) != 0 ||
        ((uintptr_t)d_row_offsets & 7u) != 0)
        return PLOGP_EINVAL;
    // one thread per (row, tile of sizes), padded to whole waves: must fit a launch
    if (cutover_items(g->view(), (int)n_tables) > ((size_t)1 << 36)) return PLOGP_ERANGE;
    return PLOGP_OK;
}

size_t plogp_cutover_rows(size_t n_tables, const plogp_grid *g)
{
    return g ? n_tables * (size_t)g->n_ops * g->n_P : 0;
}

int plogp_cutovers(plogp_grid *g, size_t n_tables, const plogp_cell *d_cells, int key_mode,
                   uint64_t *d_row_offsets, plogp_run *d_runs, size_t runs_capacity, void *stream)
{
    int rc = check_cutover_args(g, n_tables, d_cells, key_mode, d_row_offsets, d_runs, runs_capacity);
    if (rc != PLOGP_OK) return rc;
    if ((rc = ensure_init()) != PLOGP_OK) return rc;
    if ((rc = ensure_cut_scratch(g, n_tables)) != PLOGP_OK) return rc;
    HIP_TRY(launch_cutovers(g->view(), (int)n_tables, reinterpret_cast<const plogp_cell_dev *>(d_cells),
                            key_mode, g->cut, d_row_offsets, d_runs, runs_capacity,
                            (hipStream_t)stream));
    return PLOGP_OK;
}

int plogp_cutovers_profile(plogp_grid *g, size_t n_tables, const plogp_cell *d_cells, int key_mode,
                           uint64_t *d_row_offsets, plogp_run *d_runs, size_t runs_capacity,
                           void *stream, int reps, float *stage_ms_out)
{
    if (!stage_ms_out || reps < 1 || reps > 10000) return PLOGP_EINVAL;
    int rc = check_cutover_args(g, n_tables, d_cells, key_mode, d_row_offsets, d_runs, runs_capacity);
    if (rc != PLOGP_OK) return rc;
    if ((rc = ensure_init()) != PLOGP_OK) return rc;
    if ((rc = ensure_cut_scratch(g, n_tables)) != PLOGP_OK) return rc;
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    hipError_t e = hipSuccess;
    for (int i = 0; i < 4 && e == hipSuccess; ++i) e = hipEventCreate(&ev[i]);
    if (e == hipSuccess)
        e = launch_cutovers(g->view(), (int)n_tables, reinterpret_cast<const plogp_cell_dev *>(d_cells),
                            key_mode, g->cut, d_row_offsets, d_runs, runs_capacity,
                            (hipStream_t)stream, ev, reps);
    if (e == hipSuccess) e = hipEventSynchronize(ev[3]);
    float ms[3] = {0.f, 0.f, 0.f};
    for (int i = 0; i < 3 && e == hipSuccess; ++i) {
        e = hipEventElapsedTime(&ms[i], ev[i], ev[i + 1]);
        ms[i] /= (float)reps;
    }
    for (int i = 0; i < 4; ++i)
        if (ev[i]) (void)hipEventDestroy(ev[i]);
    if (e != hipSuccess) return device_error(e);
    for (int i = 0; i < 3; ++i) stage_ms_out[i] = ms[i];
    return PLOGP_OK;
}

static int score_common(const plogp_table *t, size_t table_index, plogp_grid *g, const double *d_meas,
                        const uint32_t *d_seg, double *d_pred, plogp_verdict *d_verdict,
                        plogp_strategy_score *d_scores, void *stream, int reps, float *stage_ms_out)
{
    if (!t || !g || !d_meas || !d_pred || !d_verdict || !d_scores) return PLOGP_EINVAL;
    if (table_index >= t->n_tables) return PLOGP_EINVAL;
    if ((g->mask & 0x224u) != 0 && !d_seg) return PLOGP_EINVAL;
    if (((uintptr_t)d_verdict & 15u) != 0 || ((uintptr_t)d_scores & 15u) != 0 ||
        ((uintptr_t)d_meas & 7u) != 0 || ((uintptr_t)d_pred & 7u) != 0 || ((uintptr_t)d_seg & 3u) != 0)
        return PLOGP_EINVAL;
    int rc = ensure_init();
    if (rc != PLOGP_OK) return rc;
    if ((rc = ensure_scratch(g, 1, t->n)) != PLOGP_OK) return rc;
    if (!g->score_rows) {
        hipError_t e = hipMalloc((void **)&g->score_rows, (size_t)PLOGP_N_STRATEGIES * g->n_m * 2 * sizeof(double));
        if (e != hipSuccess) {
            g->score_rows = nullptr;
            if (e == hipErrorOutOfMemory) { (void)hipGetLastError(); return PLOGP_ENOMEM; }
            return device_error(e);
        }
    }
    DeviceTables T1 = t->view();            // the one table
    T1.x += table_index * t->n;
    T1.y += table_index * t->n;
    T1.slope += table_index * t->n;
    T1.L += table_index;
    T1.n_tables = 1;
    T1.shared_x = 0;
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    hipError_t e = hipSuccess;
    if (stage_ms_out)
        for (int i = 0; i < 4 && e == hipSuccess; ++i) e = hipEventCreate(&ev[i]);
    if (e == hipSuccess)
        e = launch_score(T1, g->view(), g->scratch, g->score_rows, d_meas, d_seg, d_pred, d_verdict,
                         d_scores, (hipStream_t)stream, stage_ms_out ? ev : nullptr, reps);
    if (stage_ms_out) {
        if (e == hipSuccess) e = hipEventSynchronize(ev[3]);
        for (int i = 0; i < 3 && e == hipSuccess; ++i) {
            float ms = 0.f;
            e = hipEventElapsedTime(&ms, ev[i], ev[i + 1]);
            stage_ms_out[i] = ms / (float)reps;
        }
        for (int i = 0; i < 4; ++i)
            if (ev[i]) (void)hipEventDestroy(ev[i]);
    }
    if (e != hipSuccess) return device_error(e);
    return PLOGP_OK;
}

size_t plogp_score_strategies(const plogp_grid *g)
{
    size_t n = 0;
    if (g)
        for (int id = 0; id < PLOGP_N_STRATEGIES; ++id) n += (g->mask >> id) & 1u;
    return n;
}

int plogp_score_grid(const plogp_table *t, size_t table_index, plogp_grid *g, const double *d_meas,
                     const uint32_t *d_seg, double *d_pred, plogp_verdict *d_verdict,
                     plogp_strategy_score *d_scores, void *stream)
{
    return score_common(t, table_index, g, d_meas, d_seg, d_pred, d_verdict, d_scores, stream, 1, nullptr);
}

int plogp_score_grid_profile(const plogp_table *t, size_t table_index, plogp_grid *g,
                             const double *d_meas, const uint32_t *d_seg, double *d_pred,
                             plogp_verdict *d_verdict, plogp_strategy_score *d_scores, void *stream,
                             int reps, float *stage_ms_out)
{
    if (!stage_ms_out || reps < 1 || reps > 10000) return PLOGP_EINVAL;
    return score_common(t, table_index, g, d_meas, d_seg, d_pred, d_verdict, d_scores, stream, reps,
                        stage_ms_out);
}

static int robust_common(const plogp_grid *g, size_t n_tables, const plogp_cell *d_cells, int key_mode,
                         uint32_t *d_agree, double *d_max_dev, uint32_t *d_table_agree, void *stream,
                         int reps, float *ms_out)
{
    if (!g || !d_cells || !d_agree || n_tables < 1 || n_tables > (1u << 24)) return PLOGP_EINVAL;
    if (key_mode != PLOGP_KEY_STRATEGY && key_mode != PLOGP_KEY_STRATEGY_AND_SEGMENT) return PLOGP_EINVAL;
    if (((uintptr_t)d_cells & 15u) != 0 || ((uintptr_t)d_agree & 3u) != 0 ||
        ((uintptr_t)d_max_dev & 7u) != 0 || ((uintptr_t)d_table_agree & 3u) != 0)
        return PLOGP_EINVAL;
    const size_t cells = (size_t)g->n_ops * g->n_m * g->n_P;
    // one thread per cell position (a launch dimension), counts in 32 bits
    if (cells == 0 || cells > ((size_t)1 << 32) - 256) return PLOGP_ERANGE;
    int rc = ensure_init();
    if (rc != PLOGP_OK) return rc;
    hipEvent_t ev[2] = {nullptr, nullptr};
    hipError_t e = hipSuccess;
    if (ms_out)
        for (int i = 0; i < 2 && e == hipSuccess; ++i) e = hipEventCreate(&ev[i]);
    if (e == hipSuccess)
        e = launch_robustness(cells, (int)n_tables, reinterpret_cast<const plogp_cell_dev *>(d_cells),
                              key_mode, d_agree, d_max_dev, d_table_agree, (hipStream_t)stream,
                              ms_out ? ev : nullptr, reps);
    if (ms_out) {
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventSynchronize(ev[1]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev[0], ev[1]);
        for (int i = 0; i < 2; ++i)
            if (ev[i]) (void)hipEventDestroy(ev[i]);
        if (e == hipSuccess) *ms_out = ms / (float)reps;
    }
    if (e != hipSuccess) return device_error(e);
    return PLOGP_OK;
}

int plogp_robustness(const plogp_grid *g, size_t n_tables, const plogp_cell *d_cells, int key_mode,
                     uint32_t *d_agree, double *d_max_dev, uint32_t *d_table_agree, void *stream)
{
    return robust_common(g, n_tables, d_cells, key_mode, d_agree, d_max_dev, d_table_agree, stream, 1,
                         nullptr);
}

int plogp_robustness_profile(const plogp_grid *g, size_t n_tables, const plogp_cell *d_cells,
                             int key_mode, uint32_t *d_agree, double *d_max_dev,
                             uint32_t *d_table_agree, void *stream, int reps, float *ms_out)
{
    if (!ms_out || reps < 1 || reps > 10000) return PLOGP_EINVAL;
    return robust_common(g, n_tables, d_cells, key_mode, d_agree, d_max_dev, d_table_agree, stream, reps,
                         ms_out);
}

}  // extern "C"
