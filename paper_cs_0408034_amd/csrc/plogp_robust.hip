// gfx950 kernels of the decision-robustness summary: a batch of decision
// tables over one grid, table 0 tuned from the parameters as measured and the
// others from perturbed copies; per cell, how many of the others hold the
// decision of table 0 and how far their predicted time moves (paper, Section 4
// and the conclusion: the deviations of the predictions did not change the
// technique that is selected).
//
// Bound by HBM reads: every 16-byte record of every table is read once.  A
// thread owns one cell position and walks a slice of the tables (lanes over
// consecutive cells: a wave reads 1 KB runs); slices of tables go to different
// workgroups so that a small grid still fills the chip, and the partial counts
// meet in integer atomics (any order gives the same value; the maximum of
// non-negative doubles is the maximum of their bit patterns).
#include "plogp_internal.hpp"

namespace plogp {
namespace {

typedef unsigned long long u64;

struct RobustShape {
    u64 cells;        // records per table
    int n_tables;
    int t_chunk;      // tables per workgroup slice
    int strict;       // 1: the decision includes the segment size
};

typedef double f64x2_t __attribute__((ext_vector_type(2)));

__global__ void __launch_bounds__(256) k_robust_clear(RobustShape R, uint32_t *agree, u64 *max_dev,
                                                      uint32_t *table_agree)
{
    const u64 i = (u64)blockIdx.x * 256 + threadIdx.x;
    if (i < R.cells) {
        agree[i] = 0u;
        if (max_dev) max_dev[i] = 0ull;               // +0.0
    }
    if (table_agree && i < (u64)R.n_tables)
        table_agree[i] = i == 0 ? (uint32_t)R.cells : 0u;
}

__device__ __forceinline__ u64 key_of(const f64x2_t &rec, int strict)
{
    // second half of a record: u32 s (low), u32 strategy (high)
    const u64 k = (u64)__double_as_longlong(rec.y);
    return strict ? k : (k >> 32);
}

template <bool PER_TABLE>
__global__ void __launch_bounds__(256) k_robust(RobustShape R, const f64x2_t *__restrict__ cells,
                                                uint32_t *agree, u64 *max_dev, uint32_t *table_agree)
{
    const u64 c = (u64)blockIdx.x * 256 + threadIdx.x;
    const bool live = c < R.cells;
    const u64 cc = live ? c : R.cells - 1;            // padding lanes read a valid record
    const int t0 = 1 + (int)blockIdx.y * R.t_chunk;
    const int t1 = t0 + R.t_chunk < R.n_tables ? t0 + R.t_chunk : R.n_tables;
    const f64x2_t base = cells[cc];
    const u64 base_key = key_of(base, R.strict);
    const double base_time = base.x;
    uint32_t cnt = 0;
    double worst = 0.0;               // largest abs(T_t - T_0) of this slice (a NaN is skipped)
    const f64x2_t *p = cells + (u64)t0 * R.cells + cc;
    int t = t0;
    constexpr int U = 8;                              // records of eight tables in flight
    for (; t + U <= t1; t += U) {
        f64x2_t r[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            r[u] = __builtin_nontemporal_load(p + (u64)u * R.cells);
        p += U * R.cells;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool same = live && key_of(r[u], R.strict) == base_key;
            cnt += same ? 1u : 0u;
            const double dev = fabs(r[u].x - base_time);
            worst = dev > worst ? dev : worst;
            if (PER_TABLE) {
                const u64 votes = __ballot(same);
                if ((threadIdx.x & 63) == 0 && votes)
                    atomicAdd(table_agree + t + u, (uint32_t)__popcll(votes));
            }
        }
    }
    for (; t < t1; ++t) {
        const f64x2_t r = __builtin_nontemporal_load(p);
        p += R.cells;
        const bool same = live && key_of(r, R.strict) == base_key;
        cnt += same ? 1u : 0u;
        const double dev = fabs(r.x - base_time);
        worst = dev > worst ? dev : worst;
        if (PER_TABLE) {
            const u64 votes = __ballot(same);
            if ((threadIdx.x & 63) == 0 && votes)
                atomicAdd(table_agree + t, (uint32_t)__popcll(votes));
        }
    }
    if (live) {
        if (cnt)
            atomicAdd(agree + c, cnt);
        // the quotient is monotone in the difference (the divisor is the same for every
        // table), so the largest quotient is the quotient of the largest difference
        const double top = worst / base_time;
        if (max_dev && top > 0.0)
            atomicMax(max_dev + c, (u64)__double_as_longlong(top));
    }
}

}  // namespace

hipError_t launch_robustness(size_t cells, int n_tables, const plogp_cell_dev *d_cells, int key_mode,
                             uint32_t *d_agree, double *d_max_dev, uint32_t *d_table_agree,
                             hipStream_t st)
{
    RobustShape R;
    R.cells = cells;
    R.n_tables = n_tables;
    R.strict = key_mode == 1 ? 1 : 0;
    const u64 cell_wg = (cells + 255) / 256;
    // enough workgroups to fill the chip: slices of the tables when the grid is small
    long slices = 1;
    if (n_tables > 1) {
        slices = (long)((8192 + cell_wg - 1) / cell_wg);
        if (slices > n_tables - 1) slices = n_tables - 1;
        if (slices > 65535) slices = 65535;
        if (slices < 1) slices = 1;
    }
    R.t_chunk = n_tables > 1 ? (int)((n_tables - 1 + slices - 1) / slices) : 1;
    slices = n_tables > 1 ? (n_tables - 1 + R.t_chunk - 1) / R.t_chunk : 0;
    u64 clear_items = cells > (u64)n_tables ? cells : (u64)n_tables;
    {
        hipLaunchKernelGGL(k_robust_clear, dim3((unsigned)((clear_items + 255) / 256)), dim3(256), 0, st,
                           R, d_agree, reinterpret_cast<u64 *>(d_max_dev), d_table_agree);
        if (slices > 0) {
            const f64x2_t *recs = reinterpret_cast<const f64x2_t *>(d_cells);
            if (d_table_agree)
                hipLaunchKernelGGL(k_robust<true>, dim3((unsigned)cell_wg, (unsigned)slices), dim3(256), 0,
                                   st, R, recs, d_agree, reinterpret_cast<u64 *>(d_max_dev), d_table_agree);
            else
                hipLaunchKernelGGL(k_robust<false>, dim3((unsigned)cell_wg, (unsigned)slices), dim3(256), 0,
                                   st, R, recs, d_agree, reinterpret_cast<u64 *>(d_max_dev), d_table_agree);
        }
    }
    return hipGetLastError();
}

}  // namespace plogp
