// C ABI of the pLogP tuning library (see include/plogp.h): handle management,
// argument validation and stream plumbing.  All arithmetic of the method is
// in plogp_kernels.hip; nothing here evaluates a model or interpolates g().
#include "plogp_handles.hpp"

#include <algorithm>
#include <math.h>
#include <mutex>
#include <new>
#include <vector>

using namespace plogp;

// The scratch of plogp_tune_grid_static: device memory inside the code object, one copy per
// GPU.  In host code this name stands for the symbol, not for an address: the address on
// the current device comes from hipGetSymbolAddress, once per device (static_scratch()).
static __device__ __align__(256) unsigned char scratch[PLOGP_STATIC_SCRATCH_BYTES];

namespace {

thread_local int tl_hip_error = 0;

constexpr double kTwo53 = 9007199254740992.0;
constexpr uint64_t kTwo53u = 1ull << 53;

bool g_init_done = false;
std::mutex g_init_mutex;

constexpr int kMaxDevices = 64;
void *g_static_scratch[kMaxDevices] = {};
std::mutex g_static_mutex;

int floor_log2_u32(uint32_t v) { int f = 0; while ((v >> (f + 1)) != 0) ++f; return f; }
int ceil_log2_u32(uint32_t v) { int f = floor_log2_u32(v); return ((1u << f) == v) ? f : f + 1; }

int alloc_error(hipError_t e)
{
    if (e == hipErrorOutOfMemory) { (void)hipGetLastError(); return PLOGP_ENOMEM; }
    return device_error(e);
}

}  // namespace

#define HIP_TRY(expr) PLOGP_HIP_TRY(expr)

namespace plogp {

int device_error(hipError_t e)
{
    tl_hip_error = (int)e;
    (void)hipGetLastError();   // clear the sticky error so the next call starts clean
    return PLOGP_EDEVICE;
}

// Address of the static scratch buffer on the current device (looked up on first use there).
static int static_scratch(void **out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return device_error(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_scratch[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return device_error(hipErrorInvalidSymbol);
        g_static_scratch[dev] = p;
    }
    *out = g_static_scratch[dev];
    return PLOGP_OK;
}

int ensure_init()
{
    {
        std::lock_guard<std::mutex> lock(g_init_mutex);
        if (!g_init_done) {
            int count = 0;
            HIP_TRY(hipGetDeviceCount(&count));
            if (count < 1) return device_error(hipErrorNoDevice);
            HIP_TRY(kernels_init());
            g_init_done = true;
        }
    }
    // every table load and grid creation comes through here: the static scratch buffer of
    // the device they are made on is known before the first tune call could need it
    void *p = nullptr;
    return static_scratch(&p);
}

}  // namespace plogp

plogp_table::~plogp_table()
{
    if (d_x) (void)hipFree(d_x);
    if (d_y) (void)hipFree(d_y);
    if (d_slope) (void)hipFree(d_slope);
    if (d_L) (void)hipFree(d_L);
}

DeviceGrid plogp_grid::view() const
{
    DeviceGrid g;
    g.m = d_m; g.P = d_P; g.s = d_s; g.blk_off = d_blk_off; g.blk_mask = d_blk_mask;
    g.mu = d_mu; g.m_map = d_m_map; g.n_mu = (int)n_mu;
    g.n_m = (int)n_m; g.n_P = (int)n_P; g.n_s = (int)n_s;
    g.n_blk = n_blk; g.last_terms = last_terms; g.cl_max = cl_max;
    g.s_cap = s_cap; g.mask = mask & PLOGP_MASK_ALL; g.extra = mask >> 13; g.n_ops = n_ops;
    g.need = (((mask >> 11) | (mask >> 14)) & 1u) << 11 | (((mask >> 12) | (mask >> 15)) & 1u) << 12;
    g.blk_is_prefix = n_blk > 32 ? 1 : 0;
    return g;
}

void plogp_grid::free_scratch()
{
    if (scratch_block) (void)hipFree(scratch_block);
    scratch_block = nullptr;
    scratch_bytes = 0;
}

void plogp_grid::free_cut_scratch()
{
    if (cut.counts) (void)hipFree(cut.counts);
    if (cut.local) (void)hipFree(cut.local);
    if (cut.flags) (void)hipFree(cut.flags);
    if (cut.group_total) (void)hipFree(cut.group_total);
    if (cut.ctl) (void)hipFree(cut.ctl);
    cut = CutScratch{};
    cut_tables = 0;
}

plogp_grid::~plogp_grid()
{
    free_scratch();
    free_cut_scratch();
    if (d_m) (void)hipFree(d_m);
    if (d_mu) (void)hipFree(d_mu);
    if (d_m_map) (void)hipFree(d_m_map);
    if (d_s) (void)hipFree(d_s);
    if (d_P) (void)hipFree(d_P);
    if (d_blk_off) (void)hipFree(d_blk_off);
    if (d_blk_mask) (void)hipFree(d_blk_mask);
}

namespace plogp {

int ensure_scratch_block(plogp_grid *g, size_t bytes)
{
    if (g->scratch_bytes >= bytes) return PLOGP_OK;
    // a previous call on this handle may still be running on some stream
    HIP_TRY(hipDeviceSynchronize());
    g->free_scratch();
    const hipError_t e = hipMalloc(&g->scratch_block, bytes);
    if (e != hipSuccess) {
        g->scratch_block = nullptr;
        return alloc_error(e);
    }
    g->scratch_bytes = bytes;
    return PLOGP_OK;
}

int ensure_cut_scratch(plogp_grid *g, size_t n_tables)
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
        (e = hipMalloc((void **)&g->cut.group_total, (groups ? groups : 1) * sizeof(uint64_t))) != hipSuccess ||
        (e = hipMalloc((void **)&g->cut.ctl, cutover_ctl_words(g->view(), (int)n_tables) * sizeof(uint64_t))) != hipSuccess) {
        g->free_cut_scratch();
        return alloc_error(e);
    }
    g->cut_tables = n_tables;
    return PLOGP_OK;
}

int check_tune_args(const plogp_table *t, const plogp_grid *g, const plogp_cell *d_out, size_t d_out_bytes)
{
    if (!t || !g || !d_out) return PLOGP_EINVAL;
    if (((uintptr_t)d_out & 15u) != 0) return PLOGP_EINVAL;
    const size_t need = plogp_decision_table_bytes(t->n_tables, g);
    if (need == 0) return PLOGP_ERANGE;                 // the table's size does not fit a size_t
    if (d_out_bytes < need) return PLOGP_ENOSPC;
    return PLOGP_OK;
}

int check_cutover_args(const plogp_grid *g, size_t n_tables, const plogp_cell *d_cells, int key_mode,
                       const uint64_t *d_row_offsets, const plogp_run *d_runs, size_t runs_capacity)
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

int check_score_args(const plogp_table *t, size_t table_index, const plogp_grid *g, const double *d_meas,
                     const uint32_t *d_seg, const double *d_pred, const plogp_verdict *d_verdict,
                     const plogp_strategy_score *d_scores)
{
    if (!t || !g || !d_meas || !d_pred || !d_verdict || !d_scores) return PLOGP_EINVAL;
    if (table_index >= t->n_tables) return PLOGP_EINVAL;
    if ((g->mask & PLOGP_MASK_ALL) == 0) return PLOGP_EINVAL;       // no measured row is enabled
    if ((g->mask & 0x224u) != 0 && !d_seg) return PLOGP_EINVAL;
    if (((uintptr_t)d_verdict & 15u) != 0 || ((uintptr_t)d_scores & 15u) != 0 ||
        ((uintptr_t)d_meas & 7u) != 0 || ((uintptr_t)d_pred & 7u) != 0 || ((uintptr_t)d_seg & 3u) != 0)
        return PLOGP_EINVAL;
    return PLOGP_OK;
}

int check_robust_args(const plogp_grid *g, size_t n_tables, const plogp_cell *d_cells, int key_mode,
                      const uint32_t *d_agree, const double *d_max_dev, const uint32_t *d_table_agree,
                      size_t *cells_out)
{
    if (!g || !d_cells || !d_agree || n_tables < 1 || n_tables > (1u << 24)) return PLOGP_EINVAL;
    if (key_mode != PLOGP_KEY_STRATEGY && key_mode != PLOGP_KEY_STRATEGY_AND_SEGMENT) return PLOGP_EINVAL;
    if (((uintptr_t)d_cells & 15u) != 0 || ((uintptr_t)d_agree & 3u) != 0 ||
        ((uintptr_t)d_max_dev & 7u) != 0 || ((uintptr_t)d_table_agree & 3u) != 0)
        return PLOGP_EINVAL;
    const size_t cells = (size_t)g->n_ops * g->n_m * g->n_P;
    // one thread per cell position (a launch dimension), counts in 32 bits
    if (cells == 0 || cells > ((size_t)1 << 32) - 256) return PLOGP_ERANGE;
    *cells_out = cells;
    return PLOGP_OK;
}

}  // namespace plogp

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
    case PLOGP_ETOOBIG: return "job needs more scratch memory than the static buffer holds";
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
        (e = launch_slopes(h->view(), h->d_slope, nullptr)) != hipSuccess ||
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
    const uint32_t mask = d->strategy_mask & PLOGP_MASK_EVERY;
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
    if ((mask & ((1u << 11) | (1u << 14))) && (uint64_t)(Pmax - 1) > (kTwo53u - 1) / m_max) return PLOGP_ERANGE;
    if ((mask & ((1u << 12) | (1u << 15))) && m_max > ((kTwo53u - 1) >> (cl_max > 0 ? cl_max - 1 : 0)))
        return PLOGP_ERANGE;

    plogp_grid *g = new (std::nothrow) plogp_grid;
    if (!g) return PLOGP_ENOMEM;
    g->n_m = d->n_m; g->n_P = d->n_P; g->n_s = d->n_s;
    g->s_cap = d->s_cap;
    g->mask = mask;
    g->n_ops = ((mask & PLOGP_MASK_BCAST) ? 1 : 0) + ((mask & PLOGP_MASK_SCATTER) ? 1 : 0) +
               ((mask & PLOGP_MASK_GATHER) ? 1 : 0) + ((mask & PLOGP_MASK_BARRIER) ? 1 : 0);
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

    // everything above is host work; the device is first touched here
    int rc = ensure_init();
    if (rc != PLOGP_OK) {
        delete g;
        return rc;
    }
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
    if (!g) return 0;
    // n_ops <= 4 and n_m, n_P <= 2^24 each: their product fits; the table count may not
    const size_t per_table = (size_t)g->n_ops * g->n_m * g->n_P;
    if (n_tables != 0 && per_table > (SIZE_MAX / sizeof(plogp_cell)) / n_tables) return 0;
    return n_tables * per_table;
}

size_t plogp_decision_table_bytes(size_t n_tables, const plogp_grid *g)
{
    return plogp_decision_table_cells(n_tables, g) * sizeof(plogp_cell);
}

int plogp_tune_grid(const plogp_table *t, plogp_grid *g, plogp_cell *d_out, size_t d_out_bytes,
                    void *stream)
{
    int rc = check_tune_args(t, g, d_out, d_out_bytes);
    if (rc != PLOGP_OK) return rc;
    const DeviceTables T = t->view();
    const DeviceGrid G = g->view();
    TunePlan plan;
    if (!plan_tune(T, G, false, plan)) return PLOGP_ERANGE;
    if ((rc = ensure_scratch_block(g, plan.lay.total)) != PLOGP_OK) return rc;
    HIP_TRY(launch_tune(plan, T, G, bind_scratch(g->scratch_block, plan.lay),
                        reinterpret_cast<plogp_cell_dev *>(d_out), (hipStream_t)stream));
    return PLOGP_OK;
}

int plogp_tune_grid_static(const plogp_table *t, const plogp_grid *g, plogp_cell *d_out,
                           size_t d_out_bytes, void *stream)
{
    int rc = check_tune_args(t, g, d_out, d_out_bytes);
    if (rc != PLOGP_OK) return rc;
    const DeviceTables T = t->view();
    const DeviceGrid G = g->view();
    TunePlan plan;
    if (!plan_tune(T, G, false, plan)) return PLOGP_ERANGE;
    if (plan.lay.total > (size_t)PLOGP_STATIC_SCRATCH_BYTES) return PLOGP_ETOOBIG;
    void *base = nullptr;
    if ((rc = static_scratch(&base)) != PLOGP_OK) return rc;
    HIP_TRY(launch_tune(plan, T, G, bind_scratch(base, plan.lay),
                        reinterpret_cast<plogp_cell_dev *>(d_out), (hipStream_t)stream));
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
    for (int stage = 0; stage < CUT_STAGES; ++stage)
        HIP_TRY(launch_cutovers_stage(stage, g->view(), (int)n_tables,
                                      reinterpret_cast<const plogp_cell_dev *>(d_cells), key_mode, g->cut,
                                      d_row_offsets, d_runs, runs_capacity, (hipStream_t)stream));
    return PLOGP_OK;
}

size_t plogp_score_strategies(const plogp_grid *g)
{
    size_t n = 0;
    if (g)
        for (int id = 0; id < 13; ++id) n += (g->mask >> id) & 1u;      // the rows of Tables 1 and 2
    return n;
}

int plogp_score_grid(const plogp_table *t, size_t table_index, plogp_grid *g, const double *d_meas,
                     const uint32_t *d_seg, double *d_pred, plogp_verdict *d_verdict,
                     plogp_strategy_score *d_scores, void *stream)
{
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
    for (int stage = 0; stage < SCORE_STAGES; ++stage)
        HIP_TRY(launch_score_stage(stage, plan, T1, G, S, rows, d_meas, d_seg, d_pred, d_verdict, d_scores,
                                   (hipStream_t)stream));
    return PLOGP_OK;
}

int plogp_robustness(const plogp_grid *g, size_t n_tables, const plogp_cell *d_cells, int key_mode,
                     uint32_t *d_agree, double *d_max_dev, uint32_t *d_table_agree, void *stream)
{
    size_t cells = 0;
    int rc = check_robust_args(g, n_tables, d_cells, key_mode, d_agree, d_max_dev, d_table_agree, &cells);
    if (rc != PLOGP_OK) return rc;
    if ((rc = ensure_init()) != PLOGP_OK) return rc;
    HIP_TRY(launch_robustness(cells, (int)n_tables, reinterpret_cast<const plogp_cell_dev *>(d_cells),
                              key_mode, d_agree, d_max_dev, d_table_agree, (hipStream_t)stream));
    return PLOGP_OK;
}

}  // extern "C"
