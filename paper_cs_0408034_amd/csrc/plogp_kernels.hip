// gfx950 kernels of the pLogP tuning sweep.
//
// Arithmetic contract (what makes the decision table reproducible bit for
// bit): IEEE binary64, no contraction (-ffp-contract=off), a fused
// multiply-add only where __builtin_fma is written, integers (m, s, k, P-1,
// floor/ceil log2 P, j*m, 2^j*m) below 2^53 and therefore exact as doubles.
//
// The models are the rows of the paper's Table 1 (Broadcast) and Table 2
// (Scatter); g() is the measured gap of Section 2 read as piecewise linear.
#include "plogp_internal.hpp"

#include <math.h>

namespace plogp {
namespace {

typedef unsigned long long u64;

// ---------------------------------------------------------------- g()

// Table of one cluster staged in LDS: sizes, gaps, interval slopes.
struct LdsTable {
    const double *x;
    const double *y;
    const double *sl;
    int n;
};

// Index of the last sample with x <= z, 0 if z is below every sample.
__device__ __forceinline__ int last_not_above(const double *x, int n, double z)
{
    int lo = 0, len = n;
    while (len > 1) {
        const int half = len >> 1;
        lo = (x[lo + half] <= z) ? lo + half : lo;
        len -= half;
    }
    return lo;
}

// g(z), Section 2: linear inside the interval that starts at the last sample
// not above z; clamped to the first gap below the first sample; the last
// interval's line continues above the last sample (slope[n-1] = slope[n-2]).
__device__ __forceinline__ double gap_at(const LdsTable &t, double z)
{
    const int i = last_not_above(t.x, t.n, z);
    const double x0 = t.x[0];
    const double zc = z > x0 ? z : x0;
    return __builtin_fma(t.sl[i], zc - t.x[i], t.y[i]);
}

__device__ __forceinline__ double interval_slope(const double *x, const double *y, int n, int i)
{
    const int a = i < n - 1 ? i : n - 2;
    const double dy = y[a + 1] - y[a];
    const double dx = x[a + 1] - x[a];
    return dy / dx;
}

// Copies table t (sizes, gaps, slopes) from global memory into LDS.
__device__ __forceinline__ LdsTable stage_table(double *lds, const DeviceTables &T, int t)
{
    const int n = T.n;
    double *x = lds, *y = lds + n, *sl = lds + 2 * n;
    const double *gx = T.x + (size_t)t * n, *gy = T.y + (size_t)t * n;
    const double *gs = T.slope + (size_t)t * n;
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        x[i] = gx[i];
        y[i] = gy[i];
        sl[i] = gs[i];
    }
    __syncthreads();
    LdsTable tab = {x, y, sl, n};
    return tab;
}

// ---------------------------------------------------------------- integer terms

__device__ __forceinline__ int floor_log2(uint32_t P) { return 31 - __clz((int)P); }
__device__ __forceinline__ int ceil_log2(uint32_t P)
{
    return floor_log2(P) + ((P & (P - 1)) != 0 ? 1 : 0);
}

// k = ceil(m / s) for integers below 2^53: the rounded quotient of two such
// integers cannot reach or cross an integer it is not equal to (its error is
// below 1/s, the smallest possible distance), so ceil() of it is exact.
__device__ __forceinline__ double segments(u64 m, u64 s) { return ceil((double)m / (double)s); }

// ---------------------------------------------------------------- slopes (table load)

__global__ void __launch_bounds__(256) k_slopes(DeviceTables T)
{
    const int t = blockIdx.x, n = T.n;
    const double *x = T.x + (size_t)t * n, *y = T.y + (size_t)t * n;
    for (int i = threadIdx.x; i < n; i += blockDim.x)
        T.slope[(size_t)t * n + i] = interval_slope(x, y, n, i);
}

// ---------------------------------------------------------------- g() at arbitrary sizes

__global__ void __launch_bounds__(256) k_interp(DeviceTables T, int t, const u64 *z, size_t n,
                                                double *out)
{
    extern __shared__ double lds[];
    const LdsTable tab = stage_table(lds, T, t);
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        out[i] = gap_at(tab, (double)z[i]);
}

// ---------------------------------------------------------------- one strategy at n points

// sum_{j=1}^{P-1} g(j m) in the block order of SUM_BLOCK.
__device__ double chain_sum(const LdsTable &tab, u64 m, uint32_t P)
{
    double done = 0.0, run = 0.0;
    u64 z = 0;
    for (uint32_t j = 1; j <= P - 1; ++j) {
        z += m;
        run = run + gap_at(tab, (double)z);
        if (j % SUM_BLOCK == 0) {
            done = done + run;
            run = 0.0;
        }
    }
    return done + run;
}

__global__ void __launch_bounds__(256) k_eval(DeviceTables T, int t, int id, const u64 *dm,
                                              const uint32_t *dP, const u64 *ds, size_t n,
                                              double *out)
{
    extern __shared__ double lds[];
    const LdsTable tab = stage_table(lds, T, t);
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n)
        return;
    const u64 m = dm[i];
    const uint32_t P = dP[i];
    const bool seg = (id == 2 || id == 5 || id == 9);
    const u64 s = seg ? ds[i] : 0;
    const u64 lim = 1ull << 53;
    bool ok = m > 0 && m < lim && P >= 2 && (!seg || (s > 0 && s <= m));
    if (ok && id == 11)
        ok = (u64)(P - 1) <= (lim - 1) / m;
    if (ok && id == 12)
        ok = m <= ((lim - 1) >> (ceil_log2(P) > 0 ? ceil_log2(P) - 1 : 0));
    if (!ok) {
        out[i] = NAN;
        return;
    }
    const double L = T.L[t];
    const double q = (double)(P - 1), fl = (double)floor_log2(P), cl = (double)ceil_log2(P);
    const double gm = gap_at(tab, (double)m);
    const double g1 = gap_at(tab, 1.0);
    const double R = __builtin_fma(3.0, L, 2.0 * g1);
    double gs = 0.0, k = 0.0;
    if (seg) {
        gs = gap_at(tab, (double)s);
        k = segments(m, s);
    }
    double r;
    switch (id) {
    case 0: case 10: r = __builtin_fma(q, gm, L); break;
    case 1: r = __builtin_fma(q, gm, R); break;
    case 2: r = __builtin_fma(q, gs * k, L); break;
    case 3: r = q * (gm + L); break;
    case 4: r = q * (gm + R); break;
    case 5: r = __builtin_fma(q, gs + L, gs * (k - 1.0)); break;
    case 6: r = cl * __builtin_fma(2.0, gm, L); break;
    case 7: r = __builtin_fma(fl, gm, cl * L); break;
    case 8: r = __builtin_fma(fl, gm, cl * R); break;
    case 9: r = __builtin_fma(fl, gs * k, cl * L); break;
    case 11: r = __builtin_fma(q, L, chain_sum(tab, m, P)); break;
    default: {
        double sum = 0.0;
        const int c = ceil_log2(P);
        for (int j = 0; j < c; ++j)
            sum = sum + gap_at(tab, (double)(m << j));
        r = __builtin_fma(cl, L, sum);
    } break;
    }
    out[i] = r;
}

// ---------------------------------------------------------------- tune, step 1: per-table and per-m terms

// One workgroup per (table, chunk of blockDim m rows).  Computes the interval
// slopes from the raw samples (chunk 0 publishes them), g(m) and the prefix
// sums over j of g(2^j m) for its rows; chunk 0 also computes g(1) and g(s).
__global__ void __launch_bounds__(256) k_prep(DeviceTables T, DeviceGrid G, Scratch S, int n_chunks)
{
    extern __shared__ double lds[];
    const int t = blockIdx.x / n_chunks, chunk = blockIdx.x % n_chunks;
    const int n = T.n;
    double *x = lds, *y = lds + n, *sl = lds + 2 * n;
    const double *gx = T.x + (size_t)t * n, *gy = T.y + (size_t)t * n;
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        x[i] = gx[i];
        y[i] = gy[i];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        const double v = interval_slope(x, y, n, i);
        sl[i] = v;
        if (chunk == 0)
            T.slope[(size_t)t * n + i] = v;
    }
    __syncthreads();
    const LdsTable tab = {x, y, sl, n};

    const int mi = chunk * blockDim.x + threadIdx.x;
    if (mi < G.n_m) {
        const u64 m = G.m[mi];
        S.gm[(size_t)t * G.n_m + mi] = gap_at(tab, (double)m);
        if (G.mask & (1u << 12)) {
            double *o = S.sum2 + ((size_t)t * G.n_m + mi) * (G.cl_max + 1);
            double acc = 0.0;
            o[0] = 0.0;
            for (int j = 0; j < G.cl_max; ++j) {
                acc = acc + gap_at(tab, (double)(m << j));
                o[j + 1] = acc;
            }
        }
    }
    if (chunk == 0) {
        if (threadIdx.x == 0)
            S.g1[t] = gap_at(tab, 1.0);
        for (int si = threadIdx.x; si < G.n_s; si += blockDim.x)
            S.gs[(size_t)t * G.n_s + si] = gap_at(tab, (double)G.s[si]);
    }
}

// ---------------------------------------------------------------- tune, step 2: Scatter-chain sum

// One lane per (m, block of SUM_BLOCK consecutive j).  The arguments j*m ascend
// inside a block, so the interval index only moves forward: one search at the
// block start, then a pointer walk.  Emits the block total and, for every P of
// the grid whose P-1 falls inside the block, the running sum at that point.
__global__ void k_chain_blocks(DeviceTables T, DeviceGrid G, Scratch S, int wg_per_table)
{
    extern __shared__ double lds[];
    const int t = blockIdx.x / wg_per_table, w = blockIdx.x % wg_per_table;
    const LdsTable tab = stage_table(lds, T, t);
    const long item = (long)w * blockDim.x + threadIdx.x;
    if (item >= (long)G.n_m * G.n_blk)
        return;
    const int b = (int)(item / G.n_m), mi = (int)(item % G.n_m);
    const int n = tab.n;
    const u64 m = G.m[mi];
    const int nterms = (b == G.n_blk - 1) ? G.last_terms : SUM_BLOCK;
    int pi = G.blk_off[b];
    const int pe = G.blk_off[b + 1];
    int next = pi < pe ? (int)(G.P[pi] - 1u) - b * SUM_BLOCK : -1;
    u64 zi = ((u64)b * SUM_BLOCK + 1) * m;
    double z = (double)zi;
    int i = last_not_above(tab.x, n, z);
    double xi = tab.x[i], yi = tab.y[i], si = tab.sl[i];
    double xn = (i + 1 < n) ? tab.x[i + 1] : INFINITY;
    const double x0 = tab.x[0];
    double run = 0.0;
    double *part = S.part + ((size_t)t * G.n_m + mi) * G.n_P;
    for (int jj = 0; jj < nterms; ++jj) {
        if (jj == next) {
            part[pi] = run;
            ++pi;
            next = pi < pe ? (int)(G.P[pi] - 1u) - b * SUM_BLOCK : -1;
        }
        while (z >= xn) {
            ++i;
            xi = xn;
            yi = tab.y[i];
            si = tab.sl[i];
            xn = (i + 1 < n) ? tab.x[i + 1] : INFINITY;
        }
        const double zc = z > x0 ? z : x0;
        run = run + __builtin_fma(si, zc - xi, yi);
        zi += m;
        z = (double)zi;
    }
    if (next == nterms)
        part[pi] = run;
    if (nterms == SUM_BLOCK)
        S.blk[((size_t)t * G.n_blk + b) * G.n_m + mi] = run;
}

// One lane per (table, m): turns the block totals into their exclusive prefix
// in ascending block order (the sum of all finished blocks before block b).
__global__ void __launch_bounds__(256) k_chain_prefix(DeviceGrid G, Scratch S, int n_tables)
{
    const long id = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (long)n_tables * G.n_m)
        return;
    const int t = (int)(id / G.n_m), mi = (int)(id % G.n_m);
    double *p = S.blk + (size_t)t * G.n_blk * G.n_m + mi;
    double done = 0.0;
    for (int b = 0; b < G.n_blk; ++b) {
        const double tot = (b < G.n_blk - 1) ? p[(size_t)b * G.n_m] : 0.0;
        p[(size_t)b * G.n_m] = done;
        done = done + tot;
    }
}

// ---------------------------------------------------------------- tune, step 3: sweep, arg-min, write

struct Best {
    double t;
    uint32_t s;
    uint32_t id;
};

__device__ __forceinline__ void consider(Best &b, double T, uint32_t id, uint32_t s)
{
    if (T < b.t) {
        b.t = T;
        b.id = id;
        b.s = s;
    }
}

__device__ __forceinline__ void store_cell(plogp_cell_dev *p, const Best &b)
{
    union {
        plogp_cell_dev c;
        uint4 v;
    } u;
    u.c.time = b.t;
    u.c.s = b.s;
    u.c.strategy = b.id;
    *reinterpret_cast<uint4 *>(p) = u.v;
}

// One workgroup per (table, tile of TM message sizes, tile of ptw process
// counts); one lane per (m, P) cell, P fastest, so a wave writes consecutive
// 16-byte records.  The terms of the segmented rows that do not depend on P,
//   A = g(s) k, B = g(s) (k-1), C = g(s) + L,
// are staged in LDS once per (m, s) in passes of `sch` candidates.
__global__ void __launch_bounds__(1024)
k_sweep(DeviceTables T, DeviceGrid G, Scratch S, plogp_cell_dev *out, int TM, int ptw,
        int n_mtiles, int n_ptiles, int sch)
{
    extern __shared__ __align__(16) double sweep_lds[];
    double2 *AB = reinterpret_cast<double2 *>(sweep_lds);   // [TM][sch]
    double *C = sweep_lds + 2 * (size_t)TM * sch;           // [sch]
    __shared__ int wg_valid;

    int bid = blockIdx.x;
    const int pt = bid % n_ptiles;
    bid /= n_ptiles;
    const int mt = bid % n_mtiles;
    const int t = bid / n_mtiles;

    const int c = threadIdx.x;
    const int ml = c / ptw, pl = c % ptw;
    const int mi = mt * TM + ml, pi = pt * ptw + pl;
    const bool active = ml < TM && mi < G.n_m && pi < G.n_P;

    const double L = T.L[t];
    const uint32_t mask = G.mask;
    const u64 m = active ? G.m[mi] : 1;
    const uint32_t P = active ? G.P[pi] : 2;

    // number of candidates s <= min(m, s_cap) (the list ascends)
    int nv = 0;
    if (active && (mask & 0x224u)) {
        const u64 lim = m < G.s_cap ? m : G.s_cap;
        int lo = 0, hi = G.n_s;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (G.s[mid] <= lim) lo = mid + 1; else hi = mid;
        }
        nv = lo;
    }
    if (c == 0)
        wg_valid = 0;
    __syncthreads();
    if (nv > 0)
        atomicMax(&wg_valid, nv);
    __syncthreads();
    const int wg_nv = wg_valid;

    const double q = (double)(P - 1);
    const int fli = floor_log2(P), cli = ceil_log2(P);
    const double fl = (double)fli, cl = (double)cli;
    const double clL = cl * L;

    double b2 = INFINITY, b5 = INFINITY, b9 = INFINITY;
    int s2 = 0, s5 = 0, s9 = 0;
    const double *gs = S.gs + (size_t)t * G.n_s;

    for (int base = 0; base < wg_nv; base += sch) {
        const int len = min(sch, wg_nv - base);
        __syncthreads();
        for (int e = c; e < TM * len; e += blockDim.x) {
            const int r = e / len, o = e % len;
            const int rmi = mt * TM + r;
            if (rmi < G.n_m) {
                const double g = gs[base + o];
                const double k = segments(G.m[rmi], G.s[base + o]);
                AB[(size_t)r * sch + o] = make_double2(g * k, g * (k - 1.0));
            }
        }
        for (int o = c; o < len; o += blockDim.x)
            C[o] = gs[base + o] + L;
        __syncthreads();
        const int mine = min(len, nv - base);
        const double2 *ab = AB + (size_t)ml * sch;
        for (int o = 0; o < mine; ++o) {
            const double2 v = ab[o];
            const double T2 = __builtin_fma(q, v.x, L);
            const double T5 = __builtin_fma(q, C[o], v.y);
            const double T9 = __builtin_fma(fl, v.x, clL);
            if (T2 < b2) { b2 = T2; s2 = base + o; }
            if (T5 < b5) { b5 = T5; s5 = base + o; }
            if (T9 < b9) { b9 = T9; s9 = base + o; }
        }
    }
    if (!active)
        return;

    const double gm = S.gm[(size_t)t * G.n_m + mi];
    const size_t plane = (size_t)G.n_m * G.n_P;
    plogp_cell_dev *o = out + (size_t)t * G.n_ops * plane + (size_t)mi * G.n_P + pi;

    if (mask & 0x3FFu) {
        const double g1 = S.g1[t];
        const double R = __builtin_fma(3.0, L, 2.0 * g1);
        Best b = {INFINITY, 0u, 0xFFFFFFFFu};
        if (mask & (1u << 0)) consider(b, __builtin_fma(q, gm, L), 0, 0);
        if (mask & (1u << 1)) consider(b, __builtin_fma(q, gm, R), 1, 0);
        if ((mask & (1u << 2)) && nv > 0) consider(b, b2, 2, (uint32_t)G.s[s2]);
        if (mask & (1u << 3)) consider(b, q * (gm + L), 3, 0);
        if (mask & (1u << 4)) consider(b, q * (gm + R), 4, 0);
        if ((mask & (1u << 5)) && nv > 0) consider(b, b5, 5, (uint32_t)G.s[s5]);
        if (mask & (1u << 6)) consider(b, cl * __builtin_fma(2.0, gm, L), 6, 0);
        if (mask & (1u << 7)) consider(b, __builtin_fma(fl, gm, clL), 7, 0);
        if (mask & (1u << 8)) consider(b, __builtin_fma(fl, gm, cl * R), 8, 0);
        if ((mask & (1u << 9)) && nv > 0) consider(b, b9, 9, (uint32_t)G.s[s9]);
        store_cell(o, b);
        o += plane;
    }
    if (mask & 0x1C00u) {
        Best b = {INFINITY, 0u, 0xFFFFFFFFu};
        if (mask & (1u << 10)) consider(b, __builtin_fma(q, gm, L), 10, 0);
        if (mask & (1u << 11)) {
            const int blk = (int)((P - 1u) / SUM_BLOCK);
            const double done = S.blk[((size_t)t * G.n_blk + blk) * G.n_m + mi];
            const double run = S.part[((size_t)t * G.n_m + mi) * G.n_P + pi];
            consider(b, __builtin_fma(q, L, done + run), 11, 0);
        }
        if (mask & (1u << 12)) {
            const double s12 = S.sum2[((size_t)t * G.n_m + mi) * (G.cl_max + 1) + cli];
            consider(b, __builtin_fma(cl, L, s12), 12, 0);
        }
        store_cell(o, b);
    }
}

inline int round_up(int v, int to) { return (v + to - 1) / to * to; }

}  // namespace

// ---------------------------------------------------------------- launch wrappers

static const size_t kMaxTableLds = (size_t)3 * 4096 * sizeof(double);

hipError_t kernels_init()
{
    hipError_t e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_interp),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxTableLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_eval),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxTableLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_prep),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxTableLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_chain_blocks),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxTableLds);
    return e;
}

hipError_t launch_slopes(const DeviceTables &T, hipStream_t st)
{
    hipLaunchKernelGGL(k_slopes, dim3(T.n_tables), dim3(256), 0, st, T);
    return hipGetLastError();
}

hipError_t launch_interp(const DeviceTables &T, int table, const uint64_t *d_z, size_t n,
                         double *d_out, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    const size_t lds = (size_t)3 * T.n * sizeof(double);
    const unsigned blocks = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(k_interp, dim3(blocks), dim3(256), lds, st, T, table,
                       reinterpret_cast<const u64 *>(d_z), n, d_out);
    return hipGetLastError();
}

hipError_t launch_eval(const DeviceTables &T, int table, int strategy, const uint64_t *d_m,
                       const uint32_t *d_P, const uint64_t *d_s, size_t n, double *d_out,
                       hipStream_t st)
{
    if (n == 0) return hipSuccess;
    const size_t lds = (size_t)3 * T.n * sizeof(double);
    const unsigned blocks = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(k_eval, dim3(blocks), dim3(256), lds, st, T, table, strategy,
                       reinterpret_cast<const u64 *>(d_m), d_P,
                       reinterpret_cast<const u64 *>(d_s), n, d_out);
    return hipGetLastError();
}

hipError_t launch_tune(const DeviceTables &T, const DeviceGrid &G, const Scratch &S,
                       plogp_cell_dev *d_out, hipStream_t st, hipEvent_t *ev)
{
    hipError_t e;
    const size_t tab_lds = (size_t)3 * T.n * sizeof(double);
#define PLOGP_MARK(i)                                                            \
    do {                                                                         \
        if (ev && (e = hipEventRecord(ev[i], st)) != hipSuccess) return e;       \
    } while (0)

    PLOGP_MARK(0);
    const int n_chunks = (G.n_m + 255) / 256;
    hipLaunchKernelGGL(k_prep, dim3((unsigned)T.n_tables * n_chunks), dim3(256), tab_lds, st, T, G,
                       S, n_chunks);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    PLOGP_MARK(1);

    if (G.mask & (1u << 11)) {
        const int threads = tab_lds > 32768 ? 1024 : 256;
        const long items = (long)G.n_m * G.n_blk;
        const int wg_per_table = (int)((items + threads - 1) / threads);
        hipLaunchKernelGGL(k_chain_blocks, dim3((unsigned)T.n_tables * wg_per_table), dim3(threads),
                           tab_lds, st, T, G, S, wg_per_table);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        PLOGP_MARK(2);
        const long rows = (long)T.n_tables * G.n_m;
        hipLaunchKernelGGL(k_chain_prefix, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st, G,
                           S, T.n_tables);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        PLOGP_MARK(3);
    } else {
        PLOGP_MARK(2);
        PLOGP_MARK(3);
    }

    // tile shape: up to 1024 process counts per workgroup; several m rows when P is short
    const int ptw = G.n_P < 1024 ? G.n_P : 1024;
    int TM = 256 / ptw;
    if (TM < 1) TM = 1;
    if (TM > G.n_m) TM = G.n_m;
    const int threads = round_up(TM * ptw, 64);
    const int n_ptiles = (G.n_P + ptw - 1) / ptw;
    const int n_mtiles = (G.n_m + TM - 1) / TM;
    int sch = 2048 / TM;
    if (sch > G.n_s) sch = G.n_s;
    if (sch < 1) sch = 1;
    const size_t lds = ((size_t)2 * TM * sch + sch) * sizeof(double);
    hipLaunchKernelGGL(k_sweep, dim3((unsigned)T.n_tables * n_mtiles * n_ptiles), dim3(threads), lds,
                       st, T, G, S, d_out, TM, ptw, n_mtiles, n_ptiles, sch);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    PLOGP_MARK(4);
#undef PLOGP_MARK
    return hipSuccess;
}

}  // namespace plogp
