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

// g() at four points at once: the four searches run side by side, so that the
// LDS latencies of one halving step overlap (the step sequence depends on n only).
__device__ __forceinline__ void gap_at4(const LdsTable &t, const double (&z)[4], double (&g)[4])
{
    int lo[4] = {0, 0, 0, 0};
    int len = t.n;
    while (len > 1) {
        const int half = len >> 1;
        double xv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            xv[u] = t.x[lo[u] + half];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            lo[u] = xv[u] <= z[u] ? lo[u] + half : lo[u];
        len -= half;
    }
    const double x0 = t.x[0];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const double zc = z[u] > x0 ? z[u] : x0;
        g[u] = __builtin_fma(t.sl[lo[u]], zc - t.x[lo[u]], t.y[lo[u]]);
    }
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
// P >= 1: the bit length of P - 1 (__clz(0) is 32)
__device__ __forceinline__ int ceil_log2(uint32_t P) { return 32 - __clz((int)(P - 1u)); }

// k = ceil(m / s) for integers below 2^53: the rounded quotient of two such
// integers cannot reach or cross an integer it is not equal to (its error is
// below 1/s, the smallest possible distance), so ceil() of it is exact.
__device__ __forceinline__ double segments(u64 m, u64 s) { return ceil((double)m / (double)s); }

// The terms of the segmented rows of Table 1 that depend on (m, s) only:
//   k = ceil(m/s), A = g(s) k, B = g(s) (k-1), C = g(s) + L.
// k comes from one multiplication by the rounded reciprocal of s, which can be
// off by one, and one exact remainder m - k s (an fma) that corrects it.
__device__ __forceinline__ void segment_terms(double md, double sd, double rcp_s, double gs,
                                              double L, double &A, double &B, double &C)
{
    double k = ceil(md * rcp_s);
    const double r = __builtin_fma(-k, sd, md);        // exact: m - k s
    k = r > 0.0 ? k + 1.0 : (r <= -sd ? k - 1.0 : k);
    A = gs * k;
    B = gs * (k - 1.0);
    C = gs + L;
}

// Minimum of two doubles that are never NaN: a single v_min_f64 (the builtin
// adds a canonicalising v_max_f64 per operand in IEEE mode).
__device__ __forceinline__ double min_f64(double a, double b)
{
    double r;
    asm("v_min_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// ---------------------------------------------------------------- slopes (table load)

__global__ void __launch_bounds__(256) k_slopes(DeviceTables T, double *slope_out)
{
    const int t = blockIdx.x, n = T.n;
    const double *x = T.x + (size_t)t * n, *y = T.y + (size_t)t * n;
    for (int i = threadIdx.x; i < n; i += blockDim.x)
        slope_out[(size_t)t * n + i] = interval_slope(x, y, n, i);
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
    if (ok && (id == 11 || id == 14))
        ok = (u64)(P - 1) <= (lim - 1) / m;
    if (ok && (id == 12 || id == 15))
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
    case 0: case 10: case 13: r = __builtin_fma(q, gm, L); break;
    case 1: r = __builtin_fma(q, gm, R); break;
    case 2: r = __builtin_fma(q, gs * k, L); break;
    case 3: r = q * (gm + L); break;
    case 4: r = q * (gm + R); break;
    case 5: r = __builtin_fma(q, gs + L, gs * (k - 1.0)); break;
    case 6: r = cl * __builtin_fma(2.0, gm, L); break;
    case 7: r = __builtin_fma(fl, gm, cl * L); break;
    case 8: r = __builtin_fma(fl, gm, cl * R); break;
    case 9: r = __builtin_fma(fl, gs * k, cl * L); break;
    case 11: case 14: r = __builtin_fma(q, L, chain_sum(tab, m, P)); break;
    case 16: r = 2.0 * __builtin_fma(q, g1, L); break;
    case 17: r = 2.0 * __builtin_fma(fl, g1, cl * L); break;
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

constexpr int TERMS_ROWS = 64;       // rows of (m, s) pairs whose minimum of A is formed together

// An image of a double (no NaN) as an unsigned integer that orders the same way.
__device__ __forceinline__ unsigned long long ordered_bits(double v)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    return (b >> 63) ? ~b : b | 0x8000000000000000ull;
}

__device__ __forceinline__ double from_ordered_bits(unsigned long long k)
{
    return __longlong_as_double((long long)((k >> 63) ? k & 0x7FFFFFFFFFFFFFFFull : ~k));
}

// One workgroup per (table, chunk of blockDim items); a lane takes one m and
// one s.  Computes the interval slopes from the raw samples (into LDS, for its
// own lookups), g(m), the number of
// candidates that compete for m and the prefix sums over j of g(2^j m) for its
// rows, g(s) for its candidates and (first table only) the reciprocals 1/s used
// to get k = ceil(m/s) without a division per (m, s); chunk 0 also g(1).
__device__ __forceinline__ void terms_body(const DeviceTables &T, const DeviceGrid &G, const Scratch &S,
                                           int n_chunks, int n_mchunks, int with_pairs, int block_id,
                                           double *lds)
{
    // per table: n_chunks workgroups for the candidates and the (m, s) pairs, then n_mchunks
    // that only do the per-size part (0: the first kind does that part as well); the two
    // parts are about equally long chains of dependent steps, side by side they halve
    const int per_table = n_chunks + n_mchunks;
    const int t = block_id / per_table, c_in = block_id % per_table;
    const bool m_role = c_in >= n_chunks;
    const int chunk = m_role ? c_in - n_chunks : c_in;
    const bool first = chunk == 0 && !m_role;
    const int waves = (int)(blockDim.x >> 6);
    const int n = T.n;
    double *x = lds, *y = lds + n, *sl = lds + 2 * n;
    const double *gx = T.x + (size_t)t * n, *gy = T.y + (size_t)t * n;
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        x[i] = gx[i];
        y[i] = gy[i];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += blockDim.x)
        sl[i] = interval_slope(x, y, n, i);
    __syncthreads();
    const LdsTable tab = {x, y, sl, n};
    // for the sweep that runs its lanes over P: g(s) and 1/s of every candidate, for this
    // workgroup's own use below
    const bool pairs = (with_pairs & 1) != 0 && !m_role, stage_s = (with_pairs & 2) != 0;
    double *gs_l = lds + 3 * n, *rcp_l = gs_l + G.n_s;
    double *sd_l = lds + 3 * n + ((with_pairs & 1) ? 2 * G.n_s : 0);   // the candidates (exact as doubles)
    if (pairs || stage_s) {
        for (int si = threadIdx.x; si < G.n_s; si += blockDim.x) {
            const double sd = (double)G.s[si];
            if (pairs) {
                gs_l[si] = gap_at(tab, sd);
                rcp_l[si] = 1.0 / sd;
            }
            if (stage_s)
                sd_l[si] = sd;
        }
        __syncthreads();
    }

    // per message size: g(m), the number of candidates, the prefix of g(2^j m).  Groups
    // of 64 sizes are dealt to the waves of this table's workgroups.
    const int n_mw = (G.n_m + 63) / 64;
    // (wave w of chunk c takes group w * chunks + c first: few groups spread over the
    // workgroups, one wave in each, rather than filling the first of them)
    const int m_chunks = n_mchunks > 0 ? n_mchunks : n_chunks;
    const int m_step = m_chunks * waves;
    const int m_first = n_mchunks > 0 && !m_role ? n_mw : (int)(threadIdx.x >> 6) * m_chunks + chunk;
    for (int mw = m_first; mw < n_mw; mw += m_step) {
        const int mi = mw * 64 + (int)(threadIdx.x & 63);
        if (mi >= G.n_m)
            continue;
        const u64 m = G.m[mi];
        S.gm[(size_t)t * G.n_m + mi] = gap_at(tab, (double)m);
        {                              // candidates s <= min(m, s_cap): the list ascends
            const u64 lim = m < G.s_cap ? m : G.s_cap;
            int lo = 0, hi = G.n_s;
            if (stage_s) {             // from LDS: a step is not a round trip to memory
                const double limd = (double)lim;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (sd_l[mid] <= limd) lo = mid + 1; else hi = mid;
                }
            } else {
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (G.s[mid] <= lim) lo = mid + 1; else hi = mid;
                }
            }
            if (t == 0)
                S.nv[mi] = lo;
        }
        if (G.need & (1u << 12)) {
            double *o = S.sum2 + ((size_t)t * G.n_m + mi) * (G.cl_max + 1);   // [m][d]
            double acc = 0.0;
            o[0] = 0.0;
            for (int j0 = 0; j0 < G.cl_max; j0 += 4) {
                double z[4], g[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int j = j0 + u < G.cl_max ? j0 + u : G.cl_max - 1;
                    z[u] = (double)(m << j);
                }
                gap_at4(tab, z, g);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (j0 + u < G.cl_max) {
                        acc = acc + g[u];
                        o[j0 + u + 1] = acc;
                    }
                }
            }
        }
    }
    if (first && threadIdx.x == 0)
        S.g1[t] = gap_at(tab, 1.0);
    if (m_role)
        return;
    // per candidate: g(s), 1/s, C = g(s) + L; shared out over the chunks of this table
    const double L = T.L[t];
    for (int si = chunk * blockDim.x + threadIdx.x; si < G.n_s; si += n_chunks * blockDim.x) {
        const double sd = (double)G.s[si];
        const double gs = gap_at(tab, sd);
        S.gs[(size_t)t * G.n_s + si] = gs;
        S.segC[(size_t)t * G.n_s + si] = gs + L;
        if (t == 0)
            S.rcp[si] = 1.0 / sd;
    }
    // per (m, s): A = g(s) k and B = g(s)(k-1) for the sweep that runs its lanes over P
    // (there they are wave-uniform), +inf where s does not compete; per m the minimum of A
    // over the candidates (rows 2 and 9 of Table 1 are monotone in A).  A chunk takes whole
    // rows of (m, s) pairs, TERMS_ROWS at a time, and forms the minima in LDS on an
    // order-preserving integer image of the doubles.
    if (pairs) {
        __shared__ unsigned long long amin_l[TERMS_ROWS];
        const int rows = (G.n_m + n_chunks - 1) / n_chunks;        // rows of a chunk
        for (int r0 = chunk * rows; r0 < (chunk + 1) * rows && r0 < G.n_m; r0 += TERMS_ROWS) {
            int nr = (chunk + 1) * rows - r0;
            nr = nr < TERMS_ROWS ? nr : TERMS_ROWS;
            nr = nr < G.n_m - r0 ? nr : G.n_m - r0;
            if ((int)threadIdx.x < TERMS_ROWS)
                amin_l[threadIdx.x] = ordered_bits(INFINITY);
            __syncthreads();
            for (int e = threadIdx.x; e < nr * G.n_s; e += blockDim.x) {
                const int ml = e / G.n_s, si = e % G.n_s;
                const int mi = r0 + ml;
                const u64 m = G.m[mi], sv = G.s[si];
                const u64 lim = m < G.s_cap ? m : G.s_cap;
                double A = INFINITY, B = INFINITY, C;
                if (sv <= lim) {
                    segment_terms((double)m, (double)sv, rcp_l[si], gs_l[si], L, A, B, C);
                    atomicMin(&amin_l[ml], ordered_bits(A));
                }
                const size_t o = ((size_t)t * G.n_m + mi) * G.n_s + si;
                S.segA[o] = A;
                S.segB[o] = B;
            }
            __syncthreads();
            if ((int)threadIdx.x < nr)
                S.amin[(size_t)t * G.n_m + r0 + threadIdx.x] = from_ordered_bits(amin_l[threadIdx.x]);
            __syncthreads();
        }
    }
}

__global__ void __launch_bounds__(256) k_terms(DeviceTables T, DeviceGrid G, Scratch S, int n_chunks,
                                               int n_mchunks, int with_pairs)
{
    extern __shared__ double lds[];
    terms_body(T, G, S, n_chunks, n_mchunks, with_pairs, (int)blockIdx.x, lds);
}

// ---------------------------------------------------------------- tune, step 2: Scatter-chain sum

// sum_{j=1}^{P-1} g(j m) (Table 2, chain row).  One lane per message size; a
// lane walks U consecutive blocks of SUM_BLOCK terms side by side (they
// are independent chains of additions, so their instructions interleave and
// hide each other's latency).  Inside a chain the arguments j*m ascend, so the
// interval of the table only moves forward: one search at the start, then a
// pointer walk that keeps d = j*m - x_i (exact: integers below 2^53) and the
// interval width, so a term costs an add, a compare, an fma and the
// accumulation.  Sizes below the first sample fall into a virtual interval of
// slope 0 and gap y_0 (the clamp).  Emits each block total and, for every P of
// the grid whose P-1 falls inside a block, the running sum at that point.

typedef double f64x2 __attribute__((ext_vector_type(2)));

// The table as the chain walk sees it, in LDS, as intervals.  Interval 0 is
// virtual: [0, x_0) with gap y_0 and slope 0 (the clamp below the first
// sample); interval i + 1 starts at sample i; the last one never ends (its
// width is +inf) and starts of +inf follow it.
struct ChainCtx {
    const f64x2 *YS;      // [n + 2] {gap at the start of the interval, slope}
    const double *X;      // [n + 6] interval starts
    const double *W;      // [n + 2] interval widths
    int n;                // samples of the table
    int n_blk;
    size_t n_m;
    const u64 *blk_mask;
    const int *blk_off;
};

// Intervals of U sizes at once: for each the number of samples not above it
// (0 = the virtual interval).  The searches run side by side, so that the LDS
// latencies of one halving step overlap.
template <int U>
__device__ __forceinline__ void chain_locate(const double *X, int n, const double (&z)[U], int (&i)[U])
{
#pragma unroll
    for (int c = 0; c < U; ++c)
        i[c] = 0;
    for (int len = n; len > 1;) {
        const int half = len >> 1;
        double xv[U];
#pragma unroll
        for (int c = 0; c < U; ++c)
            xv[c] = X[1 + i[c] + half];
#pragma unroll
        for (int c = 0; c < U; ++c)
            i[c] = xv[c] <= z[c] ? i[c] + half : i[c];
        len -= half;
    }
    const double x_first = X[1];
#pragma unroll
    for (int c = 0; c < U; ++c)
        i[c] += z[c] >= x_first ? 1 : 0;
}

// Dense part of the table (small j): after moving into interval i the size is
// still at or past its end (d >= w), i.e. several intervals on.  Looks four
// intervals ahead a few times, then searches the rest of the table for the size
// itself (exact: integers below 2^53).  Leaves i, d and the interval's terms.
__device__ __forceinline__ void chain_skip_ahead(const ChainCtx &C, int &i, double &d, double &w,
                                                 double &yi, double &si)
{
    const double *X = C.X;
    double xb = X[i + 1];         // end of interval i
    double e = d - w;             // size - end of interval i
    int hops = 0;
    for (;;) {
        const double r1 = X[i + 2] - xb, r2 = X[i + 3] - xb;
        const double r3 = X[i + 4] - xb, r4 = X[i + 5] - xb;
        if (e >= r4) {
            if (++hops == 3) {
                const double z[1] = {xb + e};
                int iz[1];
                chain_locate<1>(X, C.n, z, iz);
                i = iz[0];
                d = z[0] - X[i];
                break;
            }
            i += 4;
            e -= r4;
            xb += r4;
            continue;
        }
        const int c = (e >= r1 ? 1 : 0) + (e >= r2 ? 1 : 0) + (e >= r3 ? 1 : 0);
        const double lo = c == 0 ? 0.0 : (c == 1 ? r1 : (c == 2 ? r2 : r3));
        d = e - lo;
        i += 1 + c;
        break;
    }
    const f64x2 ys = C.YS[i];
    w = C.W[i];
    yi = ys.x;
    si = ys.y;
}

// U consecutive blocks from block b0 on, walked side by side for the size m of
// this lane.  part: this size's row of in-block partial sums; tot: its column of
// block totals.
template <int U>
__device__ __forceinline__ void chain_walk(const ChainCtx &C, int b0, u64 m, double *part, double *tot)
{
    const int n = C.n;
    const int n_act = C.n_blk - b0 < U ? C.n_blk - b0 : U;      // chains that have a block
    const double md = (double)m;
    // per chain (wave-uniform): the points of its block at which some grid P needs the
    // running sum (bit r: after r terms), and where the next such sum goes
    u64 wanted[U], any_wanted = 0;
    int pi[U];
#pragma unroll
    for (int c = 0; c < U; ++c) {
        wanted[c] = c < n_act ? C.blk_mask[b0 + c] : 0ull;
        pi[c] = c < n_act ? C.blk_off[b0 + c] : 0;
        any_wanted |= wanted[c];
    }
    // A chain without a block repeats the first one and is not stored.
    double z0[U];
    int i[U];
#pragma unroll
    for (int c = 0; c < U; ++c)
        z0[c] = (double)(((u64)(c < n_act ? b0 + c : b0) * SUM_BLOCK + 1) * m);
    chain_locate<U>(C.X, n, z0, i);
    double d[U], w[U], yi[U], si[U], run[U];
    bool beyond = true;         // every chain already above the last sample
#pragma unroll
    for (int c = 0; c < U; ++c) {
        d[c] = z0[c] - C.X[i[c]];         // d = z - start of the interval (exact)
        w[c] = C.W[i[c]];
        const f64x2 ys = C.YS[i[c]];
        yi[c] = ys.x;
        si[c] = ys.y;
        run[c] = 0.0;
        beyond = beyond && i[c] == n;
    }
    // Above the last sample nothing is crossed any more: when every size of the wave is
    // there already, the walk needs no comparison at all.
    const bool no_crossing = __ballot(!beyond) == 0;
    int jj = 0;
    for (;;) {
        // run without any bookkeeping up to the next point where a sum is wanted
        const int hit = any_wanted != 0 ? __builtin_ctzll(any_wanted) : SUM_BLOCK;
        if (no_crossing) {
            for (; jj < hit; ++jj) {
#pragma unroll
                for (int c = 0; c < U; ++c) {
                    run[c] = run[c] + __builtin_fma(si[c], d[c], yi[c]);
                    d[c] += md;
                }
            }
        }
        for (; jj < hit; ++jj) {
            bool cross[U], any_cross = false;
#pragma unroll
            for (int c = 0; c < U; ++c) {
                cross[c] = d[c] >= w[c];
                any_cross = any_cross || cross[c];
            }
            if (any_cross) {            // some chain enters its next interval
#pragma unroll
                for (int c = 0; c < U; ++c) {
                    if (cross[c]) {
                        d[c] -= w[c];
                        ++i[c];
                        const f64x2 ys = C.YS[i[c]];
                        w[c] = C.W[i[c]];
                        yi[c] = ys.x;
                        si[c] = ys.y;
                        if (d[c] >= w[c])
                            chain_skip_ahead(C, i[c], d[c], w[c], yi[c], si[c]);
                    }
                }
            }
#pragma unroll
            for (int c = 0; c < U; ++c) {
                run[c] = run[c] + __builtin_fma(si[c], d[c], yi[c]);
                d[c] += md;
            }
        }
        if (hit == SUM_BLOCK)
            break;
#pragma unroll
        for (int c = 0; c < U; ++c) {
            if ((wanted[c] >> hit) & 1ull) {
                part[pi[c]] = run[c];
                ++pi[c];
            }
        }
        any_wanted &= any_wanted - 1;
    }
#pragma unroll
    for (int c = 0; c < U; ++c)
        if (c < n_act && b0 + c < C.n_blk - 1)     // the last block is never complete
            tot[(size_t)(b0 + c) * C.n_m] = run[c];
}

// One block whose consecutive sizes j m lie many intervals apart (small j on a
// table with many samples): every term gets its own search of the table, four
// terms side by side; the terms are added in ascending j as everywhere.
__device__ __forceinline__ void chain_search_block(const ChainCtx &C, int b, u64 m, double *part,
                                                   double *tot)
{
    constexpr int V = 4;
    const u64 wanted = C.blk_mask[b];
    int pi = C.blk_off[b];
    const u64 j0 = (u64)b * SUM_BLOCK + 1;
    double run = 0.0;
    for (int r0 = 0; r0 < SUM_BLOCK; r0 += V) {
        double z[V], g[V];
        int i[V];
#pragma unroll
        for (int c = 0; c < V; ++c)
            z[c] = (double)((j0 + r0 + c) * m);
        chain_locate<V>(C.X, C.n, z, i);
#pragma unroll
        for (int c = 0; c < V; ++c) {
            const f64x2 ys = C.YS[i[c]];
            g[c] = __builtin_fma(ys.y, z[c] - C.X[i[c]], ys.x);
        }
#pragma unroll
        for (int c = 0; c < V; ++c) {
            if ((wanted >> (r0 + c)) & 1ull) {      // bit r: the sum after r terms is wanted
                part[pi] = run;
                ++pi;
            }
            run = run + g[c];
        }
    }
    if (b < C.n_blk - 1)
        tot[(size_t)b * C.n_m] = run;
}

// Work items of one table, in this order: (block b, group of 64 sizes mg) for the
// n_single leading blocks, one block each -- small j, where the walk crosses
// many intervals per term and an item takes longest; the first n_search of them
// search per term -- then (unit u, mg) with CHAIN_U blocks each.  The items are
// dealt to the workgroups of the table in rounds, every other round in reverse
// order, so that every workgroup gets its share of the heavy items and meets
// them first; inside a workgroup the waves take the next item of its list from
// a counter in LDS, because how long an item takes depends on how often its
// sizes cross an interval.
constexpr int CHAIN_U = 4;           // blocks walked side by side by a lane in the sparse part

__device__ __forceinline__ void chain_body(const DeviceTables &T, const DeviceGrid &G, const Scratch &S,
                                           int wg_per_table, int n_single, int n_search, int block_id,
                                           double *chain_lds)
{
    __shared__ unsigned next_item;
    const int t = block_id / wg_per_table, wg = block_id % wg_per_table;
    const int n = T.n;
    // the table as intervals, built from the raw samples (the slopes are those of the
    // tuning's first step: the same expression): YS[0..n+1] = {gap, slope}, X[0..n+5] =
    // interval starts (0, the samples, +inf ...), W = widths
    f64x2 *YS = reinterpret_cast<f64x2 *>(chain_lds);              // n + 2 entries
    double *X = chain_lds + 2 * (n + 2);                           // n + 6 entries, +inf from n + 1 on
    double *W = X + (n + 6);                                       // n + 2 entries
    {
        const double *gx = T.x + (size_t)t * n, *gy = T.y + (size_t)t * n;
        for (int i = threadIdx.x; i < n + 6; i += blockDim.x) {
            // interval i starts at sample i - 1; interval 0 is the clamp below the first sample
            const double x0 = i == 0 ? 0.0 : i <= n ? gx[i - 1] : INFINITY;
            X[i] = x0;
            if (i < n + 2) {
                f64x2 ys;
                ys.x = i == 0 ? gy[0] : i <= n ? gy[i - 1] : 0.0;
                ys.y = (i == 0 || i > n) ? 0.0 : interval_slope(gx, gy, n, i - 1);
                YS[i] = ys;
                W[i] = i < n ? gx[i] - x0 : INFINITY;
            }
        }
        if (threadIdx.x == 0)
            next_item = 0u;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int n_mg = (G.n_mu + 63) / 64;      // groups of 64 distinct sizes
    const unsigned n_single_items = (unsigned)n_single * (unsigned)n_mg;
    const unsigned n_units = (unsigned)((G.n_blk - n_single + CHAIN_U - 1) / CHAIN_U);
    const unsigned n_items = n_single_items + n_units * (unsigned)n_mg;
    const unsigned W_ = (unsigned)wg_per_table;
    ChainCtx C;
    C.YS = YS;
    C.X = X;
    C.W = W;
    C.n = n;
    C.n_blk = G.n_blk;
    C.n_m = (size_t)G.n_mu;
    C.blk_mask = G.blk_mask;
    C.blk_off = G.blk_off;
    for (;;) {
        unsigned k = 0;
        if (lane == 0)
            k = atomicAdd(&next_item, 1u);
        k = __builtin_amdgcn_readfirstlane(k);
        // round k of the deal: this workgroup's place is wg, or W_ - 1 - wg in odd rounds
        const unsigned item = k * W_ + ((k & 1u) ? W_ - 1u - (unsigned)wg : (unsigned)wg);
        if (item >= n_items)
            break;                        // later rounds lie further on still
        const bool single = item < n_single_items;
        const unsigned rest = single ? item : item - n_single_items;
        const int u = (int)(rest / (unsigned)n_mg), mg = (int)(rest % (unsigned)n_mg);
        const int mi = mg * 64 + lane;
        if (mi >= G.n_mu)
            continue;
        const u64 m = G.mu[mi];
        double *part = S.part + ((size_t)t * C.n_m + mi) * G.n_P;     // [m][P index]
        double *tot = S.blk + (size_t)t * G.n_blk * C.n_m + mi;       // [block][m]
        if (!single)
            chain_walk<CHAIN_U>(C, n_single + u * CHAIN_U, m, part, tot);
        else if (u < n_search)
            chain_search_block(C, u, m, part, tot);
        else
            chain_walk<1>(C, u, m, part, tot);
    }
}

// The same sums for a small job (few samples, about a million terms or fewer), where the
// walk above is bound by the latency of one lane's 64 dependent steps and the chip is
// nearly idle: a workgroup takes one (block, 64 sizes) item at a time; its four waves
// evaluate the 64 x 64 terms side by side, each by a search of its own (the same
// expression, so the same gaps), into LDS; one wave then adds the terms of each size in
// order, leaving the sum before every term in place; all waves write the wanted partial
// sums, a row of the output per store.
constexpr int SMALL_LD = 65;          // row stride of the 64 x 64 tile of terms

__device__ __forceinline__ void chain_small_body(const DeviceTables &T, const DeviceGrid &G,
                                                 const Scratch &S, int wg_per_table, int block_id,
                                                 double *chain_lds)
{
    const int t = block_id / wg_per_table, wg = block_id % wg_per_table;
    const int n = T.n;
    f64x2 *YS = reinterpret_cast<f64x2 *>(chain_lds);              // n + 2 entries
    double *X = chain_lds + 2 * (n + 2);                           // n + 6 entries
    double *gl = X + (n + 6);                                      // 64 rows of SMALL_LD
    const int lane = threadIdx.x & 63, wave = (int)(threadIdx.x >> 6);
    const int n_mu = G.n_mu;
    const int n_mg = (n_mu + 63) / 64;
    const int n_items = G.n_blk * n_mg;
    // the first item's size, block mask and offset are on their way while the table is staged
    u64 m_next = 0, wanted_next = 0;
    int off_next = 0;
    if (wg < n_items) {
        const int mi0 = (wg % n_mg) * 64 + lane;
        m_next = G.mu[mi0 < n_mu ? mi0 : n_mu - 1];
        wanted_next = G.blk_mask[wg / n_mg];
        off_next = G.blk_off[wg / n_mg];
    }
    {
        const double *gx = T.x + (size_t)t * n, *gy = T.y + (size_t)t * n;
        for (int i = threadIdx.x; i < n + 6; i += blockDim.x) {
            X[i] = i == 0 ? 0.0 : i <= n ? gx[i - 1] : INFINITY;
            if (i < n + 2) {
                f64x2 ys;
                ys.x = i == 0 ? gy[0] : i <= n ? gy[i - 1] : 0.0;
                ys.y = (i == 0 || i > n) ? 0.0 : interval_slope(gx, gy, n, i - 1);
                YS[i] = ys;
            }
        }
    }
    __syncthreads();
    for (int item = wg; item < n_items; item += wg_per_table) {
        const int b = item / n_mg, mg = item % n_mg;
        const int mi = mg * 64 + lane;
        const u64 m = m_next, wanted = wanted_next;
        const int off = off_next;
        if (item + wg_per_table < n_items) {
            const int nxt = item + wg_per_table;
            const int mi1 = (nxt % n_mg) * 64 + lane;
            m_next = G.mu[mi1 < n_mu ? mi1 : n_mu - 1];
            wanted_next = G.blk_mask[nxt / n_mg];
            off_next = G.blk_off[nxt / n_mg];
        }
        const u64 j0 = (u64)b * SUM_BLOCK + 1 + (u64)wave * 16;     // this wave's 16 terms
#pragma unroll
        for (int r0 = 0; r0 < 16; r0 += 8) {                        // eight searches side by side
            double z[8];
            int i[8];
#pragma unroll
            for (int c = 0; c < 8; ++c)
                z[c] = (double)((j0 + r0 + c) * m);
            chain_locate<8>(X, n, z, i);
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const f64x2 ys = YS[i[c]];
                gl[(wave * 16 + r0 + c) * SMALL_LD + lane] = __builtin_fma(ys.y, z[c] - X[i[c]], ys.x);
            }
        }
        __syncthreads();
        if (wave == 0) {
            double run = 0.0;
            for (int r0 = 0; r0 < SUM_BLOCK; r0 += 8) {
                double g[8];
#pragma unroll
                for (int c = 0; c < 8; ++c)
                    g[c] = gl[(r0 + c) * SMALL_LD + lane];
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    gl[(r0 + c) * SMALL_LD + lane] = run;          // the sum before term r0 + c
                    run = run + g[c];
                }
            }
            if (mi < n_mu && b < G.n_blk - 1)
                S.blk[((size_t)t * G.n_blk + b) * n_mu + mi] = run;
        }
        __syncthreads();
        {
            // lane r holds term r's place: bit r of the mask = the sum before term r is wanted
            const bool want = ((wanted >> lane) & 1ull) != 0;
            const int at = off + __popcll(wanted & ((1ull << lane) - 1ull));
            for (int row = wave; row < 64; row += 4) {
                const int mrow = mg * 64 + row;
                if (mrow < n_mu && want)
                    S.part[((size_t)t * n_mu + mrow) * G.n_P + at] = gl[lane * SMALL_LD + row];
            }
        }
        __syncthreads();
    }
}

// terms_mode >= 0: a workgroup that has run out of sums goes on with its share of the tuning's
// first step (as chunk blockIdx.x of wg_per_table per table), in the same LDS: for a big
// table that step is a few dependent lookups per workgroup, which fit in the time the
// workgroups wait for the slowest of them anyway, and a launch less.
__global__ void k_chain_blocks(DeviceTables T, DeviceGrid G, Scratch S, int wg_per_table,
                               int n_single, int n_search, int terms_mode)
{
    extern __shared__ __align__(16) double chain_lds[];
    chain_body(T, G, S, wg_per_table, n_single, n_search, (int)blockIdx.x, chain_lds);
    if (terms_mode >= 0) {
        __syncthreads();                  // every wave is done with the table as intervals
        terms_body(T, G, S, wg_per_table, 0, terms_mode, (int)blockIdx.x, chain_lds);
    }
}

// The Scatter-chain sums of one (table, distinct m) in one workgroup, for tables of few
// samples and sums of few blocks: what k_chain_blocks and k_chain_prefix leave in device
// memory (the in-block sums at the grid's process counts, and the totals of the finished
// blocks or their prefix), without a lane that walks a block alone.  A thread evaluates 16
// consecutive terms g(j m) (one search, then a walk: the sizes ascend), into a tile in LDS;
// a lane per block adds its 64 terms in order and leaves the sum before every term in
// place; one lane adds the block totals in order; all threads write the sums out, the
// process counts along the lanes.
constexpr int CROW_THREADS = 256;
constexpr int CROW_MAX_BLK = 96;         // 6144 terms at most
constexpr int CROW_TPT = 16;             // consecutive terms per thread
constexpr int CROW_LD = SUM_BLOCK + SUM_BLOCK / CROW_TPT + 1;     // 69: a block's row in the tile

// term r (0-based) sits at r + r / 64 + r / 16: rows of 69, so that neither the threads
// that write runs of 16 nor the lanes that read one row each meet in a bank
__device__ __forceinline__ int crow_at(int r) { return r + r / SUM_BLOCK + r / CROW_TPT; }

static size_t chain_row_lds(int n, int n_blk)
{
    return ((size_t)3 * n + (size_t)n_blk * CROW_LD + 2 * CROW_MAX_BLK) * sizeof(double);
}

__device__ __forceinline__ void chain_row_body(const DeviceTables &T, const DeviceGrid &G, const Scratch &S,
                                               int block_id, double *lds)
{
    const int n = T.n, n_blk = G.n_blk, n_mu = G.n_mu, n_P = G.n_P;
    const int tid = threadIdx.x;
    const int t = block_id / n_mu, mu_i = block_id % n_mu;
    double *x = lds, *y = x + n, *sl = y + n;
    double *pre = sl + n;                                  // the terms, then the sums before each
    double *tot = pre + (size_t)n_blk * CROW_LD, *done = tot + CROW_MAX_BLK;
    const u64 m = G.mu[mu_i];
    const uint32_t P_first = tid < n_P ? G.P[tid] : 2u;    // asked for now, used at the very end
    {
        const double *gx = T.x + (size_t)t * n, *gy = T.y + (size_t)t * n;
        for (int i = tid; i < n; i += CROW_THREADS) {
            x[i] = gx[i];
            y[i] = gy[i];
        }
        __syncthreads();
        for (int i = tid; i < n; i += CROW_THREADS)
            sl[i] = interval_slope(x, y, n, i);
        __syncthreads();
    }
    const double md = (double)m, x0 = x[0];
    const int n_terms = SUM_BLOCK * (n_blk - 1) + G.last_terms;
    for (int r0 = tid * CROW_TPT; r0 < n_blk * SUM_BLOCK; r0 += CROW_THREADS * CROW_TPT) {
        // g((r + 1) m) for r = r0 .. r0 + 15: the same expression as gap_at, with the interval
        // carried along (i: the last sample not above the size, 0 below the first)
        double z = (double)((u64)(r0 + 1) * m);
        int i = last_not_above(x, n, z);
        double xi = x[i], yi = y[i], si = sl[i];
        double xn = i + 1 < n ? x[i + 1] : INFINITY;
#pragma unroll 4
        for (int k = 0; k < CROW_TPT; ++k) {
            double v = 0.0;
            if (r0 + k < n_terms) {
                while (z >= xn) {
                    ++i;
                    xi = xn;
                    yi = y[i];
                    si = sl[i];
                    xn = i + 1 < n ? x[i + 1] : INFINITY;
                }
                const double zc = z > x0 ? z : x0;
                v = __builtin_fma(si, zc - xi, yi);
            }
            pre[crow_at(r0 + k)] = v;
            z += md;                                       // exact: integers below 2^53
        }
    }
    __syncthreads();
    if (tid < n_blk) {
        // sixteen terms at a time: read, add in order, write the sums before each
        double *p = pre + tid * CROW_LD;
        double run = 0.0;
        for (int r0 = 0; r0 < SUM_BLOCK; r0 += CROW_TPT) {
            double v[CROW_TPT];
            double *q = p + r0 + r0 / CROW_TPT;
#pragma unroll
            for (int u = 0; u < CROW_TPT; ++u)
                v[u] = q[u];
#pragma unroll
            for (int u = 0; u < CROW_TPT; ++u) {
                q[u] = run;
                run = run + v[u];
            }
        }
        tot[tid] = run;
    } else if (tid < CROW_MAX_BLK) {
        tot[tid] = 0.0;
    }
    __syncthreads();
    if (tid == 0) {
        // the finished blocks, in ascending order; sixteen totals per round trip to LDS
        double acc = 0.0;
        for (int b0 = 0; b0 < n_blk; b0 += 16) {
            double v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u)
                v[u] = tot[b0 + u];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                done[b0 + u] = acc;
                acc = acc + v[u];
            }
        }
    }
    __syncthreads();
    const size_t row = (size_t)t * n_mu + mu_i;
    for (int pi = tid; pi < n_P; pi += CROW_THREADS) {
        const int r = (int)((pi == tid ? P_first : G.P[pi]) - 1u), blk = r / SUM_BLOCK;
        S.part[row * n_P + pi] = pre[crow_at(r)];
        if (G.blk_is_prefix)
            S.pre[row * n_P + pi] = done[blk];
    }
    if (!G.blk_is_prefix)
        for (int b = tid; b < n_blk - 1; b += CROW_THREADS)        // the last block is never complete
            S.blk[((size_t)t * n_blk + b) * n_mu + mu_i] = tot[b];
}

__global__ void __launch_bounds__(CROW_THREADS) k_chain_row(DeviceTables T, DeviceGrid G, Scratch S)
{
    extern __shared__ double lds[];
    chain_row_body(T, G, S, (int)blockIdx.x, lds);
}

// The terms and the sums above in one launch, side by side: both are short chains of
// dependent steps.  The (few) terms workgroups come first, so that they are on the chip at
// once.
__global__ void __launch_bounds__(CROW_THREADS) k_terms_chain_row(DeviceTables T, DeviceGrid G, Scratch S,
                                                                  int terms_wg, int n_chunks, int n_mchunks,
                                                                  int with_pairs)
{
    extern __shared__ __align__(16) double both_lds[];
    if ((int)blockIdx.x < terms_wg)
        terms_body(T, G, S, n_chunks, n_mchunks, with_pairs, (int)blockIdx.x, both_lds);
    else
        chain_row_body(T, G, S, (int)blockIdx.x - terms_wg, both_lds);
}

// Both first steps in one launch: they do not depend on each other (each stages the
// table from the raw samples), so the workgroups of the chain sums (the longer job, first
// in the grid) and those of the terms run side by side.  For tables small enough that
// workgroups of both kinds share a CU.
__global__ void __launch_bounds__(256) k_terms_chain(DeviceTables T, DeviceGrid G, Scratch S, int n_chain_wg,
                                                     int wg_per_table, int n_single, int n_search,
                                                     int n_chunks, int n_mchunks, int with_pairs)
{
    extern __shared__ __align__(16) double both_lds[];
    if ((int)blockIdx.x < n_chain_wg) {
        if (n_single < 0)                 // a small job: terms by search, side by side
            chain_small_body(T, G, S, wg_per_table, (int)blockIdx.x, both_lds);
        else
            chain_body(T, G, S, wg_per_table, n_single, n_search, (int)blockIdx.x, both_lds);
    } else
        terms_body(T, G, S, n_chunks, n_mchunks, with_pairs, (int)blockIdx.x - n_chain_wg, both_lds);
}

// Turns the block totals of PFX_M message sizes into their exclusive prefix in
// ascending block order (the sum of all finished blocks before block b) and
// writes, per process count of the grid, the prefix of the block it ends in:
// pre[m][P index], which the sweeps read side by side with the partial sums.  The sum is
// sequential per m; the workgroup moves tiles of PFX_TILE blocks through LDS
// (every thread 16 loads in flight) and the first PFX_M lanes scan a tile there.
constexpr int PFX_TILE = 256;
constexpr int PFX_M = 16;
constexpr int PFX_MAX_P = 4096;     // process counts whose block index is kept in LDS

__global__ void __launch_bounds__(256) k_chain_prefix(DeviceGrid G, Scratch S, int n_mgroups)
{
    __shared__ double tile[PFX_TILE * (PFX_M + 1)];      // [block][m], rows padded by one
    const int t = blockIdx.x / n_mgroups, mg = blockIdx.x % n_mgroups;
    const int tid = threadIdx.x;
    const int ml = tid % PFX_M, br = tid / PFX_M;        // br: 0 .. 256 / PFX_M - 1
    constexpr int ROWS = 256 / PFX_M;                    // rows of the tile loaded per pass
    const int mi = mg * PFX_M + ml;
    const bool active = mi < G.n_mu;
    const size_t n_m = (size_t)G.n_mu;       // rows: the distinct sizes
    const double *src = S.blk + (size_t)t * G.n_blk * n_m + (active ? mi : 0);
    const int full = G.n_blk - 1;                        // blocks that have a total
    double done = 0.0;
    double v[PFX_TILE / ROWS];
    auto load_tile = [&](int b0) {
#pragma unroll
        for (int k = 0; k < PFX_TILE / ROWS; ++k) {
            const int b = b0 + br + ROWS * k;
            v[k] = (active && b < full) ? src[(size_t)b * n_m] : 0.0;
        }
    };
    load_tile(0);
    // the block of every process count of the grid, kept in LDS when there are few enough:
    // writing the results out then waits for no load from device memory
    __shared__ int blk_of[PFX_MAX_P];
    const bool p_in_lds = G.n_P <= PFX_MAX_P;
    if (p_in_lds)
        for (int pi = tid; pi < G.n_P; pi += 256)
            blk_of[pi] = (int)((G.P[pi] - 1u) / SUM_BLOCK);
    // the process counts whose sums end in the current tile: P indices [off_lo, off_hi)
    const int m_valid = G.n_mu - mg * PFX_M < PFX_M ? G.n_mu - mg * PFX_M : PFX_M;   // sizes of this group
    int off_lo = G.blk_off[0];
    int off_hi = G.blk_off[PFX_TILE < G.n_blk ? PFX_TILE : G.n_blk];
    for (int b0 = 0; b0 < G.n_blk; b0 += PFX_TILE) {
#pragma unroll
        for (int k = 0; k < PFX_TILE / ROWS; ++k)
            tile[(br + ROWS * k) * (PFX_M + 1) + ml] = v[k];
        const int pi_lo = off_lo, pi_hi = off_hi;
        __syncthreads();
        // the next tile's totals and range are on their way while this one is scanned and
        // written
        if (b0 + PFX_TILE < G.n_blk) {
            load_tile(b0 + PFX_TILE);
            off_lo = off_hi;
            off_hi = G.blk_off[b0 + 2 * PFX_TILE < G.n_blk ? b0 + 2 * PFX_TILE : G.n_blk];
        }
        if (tid < PFX_M) {
            // sixteen totals at a time: read, add in order, write the sums before each (rows
            // past the last block hold zeros and are not written out below)
            const int nb = G.n_blk - b0 < PFX_TILE ? G.n_blk - b0 : PFX_TILE;
            for (int bb = 0; bb < nb; bb += 16) {
                double tot[16];
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    tot[u] = tile[(bb + u) * (PFX_M + 1) + tid];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    tile[(bb + u) * (PFX_M + 1) + tid] = done;
                    done = done + tot[u];
                }
            }
        }
        __syncthreads();
        // only the blocks in which some process count of the grid ends are wanted: the sums
        // go out per process count, pre[m][P index], a run of the output per m and store
        {
            for (int pi = pi_lo + tid; pi < pi_hi; pi += 256) {
                const int bb = (p_in_lds ? blk_of[pi] : (int)((G.P[pi] - 1u) / SUM_BLOCK)) - b0;
                // all the sums of the row first (one wait for LDS), then the stores
                double row[PFX_M];
#pragma unroll
                for (int mm = 0; mm < PFX_M; ++mm)
                    row[mm] = tile[bb * (PFX_M + 1) + mm];
                double *o = S.pre + ((size_t)t * n_m + (size_t)mg * PFX_M) * G.n_P + pi;
#pragma unroll
                for (int mm = 0; mm < PFX_M; ++mm) {
                    if (mm < m_valid)
                        o[(size_t)mm * G.n_P] = row[mm];
                }
            }
        }
        __syncthreads();
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

// A 16-byte record of an output that no kernel of the call reads again: stored with the
// non-temporal hint, so that the stream of cells does not push the tables and terms out of the
// caches (measured on the 1.97 GB table of 10 000 clusters: 5 % off the whole kernel).
__device__ __forceinline__ void stream_out(void *p, uint4 v)
{
    typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
    u32x4_t w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, reinterpret_cast<u32x4_t *>(p));
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
    stream_out(p, u.v);
}

// Broadcast: the ten rows of Table 1 in id order, strict '<' (ties: lowest id).
// t2/t5/t9 are the minima over s of the segmented rows (+inf if none), s2/s5/s9
// the segment sizes that attain them.
__device__ __forceinline__ Best decide_bcast(uint32_t mask, double q, double fl, double cl,
                                             double gm, double L, double g1, double t2,
                                             uint32_t s2, double t5, uint32_t s5, double t9,
                                             uint32_t s9)
{
    const double clL = cl * L;
    // A rendezvous row adds R - L = 2 g(1) + 2 L to its plain twin's latency term.  Gaps
    // and latencies are checked to be non-negative when a table is loaded and g(1) is the
    // first gap (size 1 is never above the first sample), so R >= L, and as rounding is
    // monotone a rendezvous row is never below its twin; with the twin enabled (lower id:
    // it also wins ties) the rendezvous row cannot be chosen and is not evaluated.
    if ((mask & 0x3FFu) == 0x3FFu) {
        // the usual case, every row enabled: rows 0, 2, 3, 5, 6, 7, 9 compete; the minimum,
        // then the lowest id that attains it (the compares do not depend on one another and
        // no partial minimum stays live)
        const double v0 = __builtin_fma(q, gm, L), v3 = q * (gm + L);
        const double v6 = cl * __builtin_fma(2.0, gm, L), v7 = __builtin_fma(fl, gm, clL);
        const double best =
            min_f64(min_f64(min_f64(v0, t2), min_f64(v3, t5)), min_f64(min_f64(v6, v7), t9));
        uint32_t id = 9u;
        id = v7 == best ? 7u : id;
        id = v6 == best ? 6u : id;
        id = t5 == best ? 5u : id;
        id = v3 == best ? 3u : id;
        id = t2 == best ? 2u : id;
        id = v0 == best ? 0u : id;
        Best b;
        b.t = best;
        b.id = id;
        b.s = id == 2u ? s2 : (id == 5u ? s5 : (id == 9u ? s9 : 0u));
        return b;
    }
    const double R = __builtin_fma(3.0, L, 2.0 * g1);   // rendezvous: 2 g(1) + 3 L
    Best b = {INFINITY, 0u, 0xFFFFFFFFu};
    // a rendezvous row (1, 4, 8) is evaluated only when its plain twin (0, 3, 7) is masked out
    if (mask & (1u << 0)) consider(b, __builtin_fma(q, gm, L), 0, 0);
    if ((mask & 3u) == 2u) consider(b, __builtin_fma(q, gm, R), 1, 0);
    if (mask & (1u << 2)) consider(b, t2, 2, s2);
    if (mask & (1u << 3)) consider(b, q * (gm + L), 3, 0);
    if ((mask & 0x18u) == 0x10u) consider(b, q * (gm + R), 4, 0);
    if (mask & (1u << 5)) consider(b, t5, 5, s5);
    if (mask & (1u << 6)) consider(b, cl * __builtin_fma(2.0, gm, L), 6, 0);
    if (mask & (1u << 7)) consider(b, __builtin_fma(fl, gm, clL), 7, 0);
    if ((mask & 0x180u) == 0x100u) consider(b, __builtin_fma(fl, gm, cl * R), 8, 0);
    if (mask & (1u << 9)) consider(b, t9, 9, s9);
    return b;
}

// Scatter: the three rows of Table 2, given the two sums for this (m, P).
__device__ __forceinline__ Best decide_scatter(uint32_t mask, double q, double cl, double gm,
                                               double L, double s11, double s12)
{
    if ((mask & 0x1C00u) == 0x1C00u) {
        // every row enabled: the minimum, then the lowest id that attains it
        const double v10 = __builtin_fma(q, gm, L), v11 = __builtin_fma(q, L, s11);
        const double v12 = __builtin_fma(cl, L, s12);
        Best b;
        b.t = min_f64(min_f64(v10, v11), v12);
        b.s = 0u;
        b.id = v10 == b.t ? 10u : (v11 == b.t ? 11u : 12u);
        return b;
    }
    Best b = {INFINITY, 0u, 0xFFFFFFFFu};
    if (mask & (1u << 10)) consider(b, __builtin_fma(q, gm, L), 10, 0);
    if (mask & (1u << 11)) consider(b, __builtin_fma(q, L, s11), 11, 0);
    if (mask & (1u << 12)) consider(b, __builtin_fma(cl, L, s12), 12, 0);
    return b;
}

// sum_{j=1}^{P-1} g(j m) for (m index mi, P index pi) from the block sums
__device__ __forceinline__ double chain_sum_of(const DeviceGrid &G, const Scratch &S, int t, int mi,
                                               int pi, uint32_t P)
{
    const size_t n_m = (size_t)G.n_mu;      // the chain sums are kept per distinct size
    mi = G.m_map[mi];
    const int blk = (int)((P - 1u) / SUM_BLOCK);
    double done;
    if (G.blk_is_prefix) {
        done = S.pre[((size_t)t * n_m + mi) * G.n_P + pi];
    } else {                           // few blocks: add the finished ones here, in ascending order
        const double *tot = S.blk + (size_t)t * G.n_blk * n_m + mi;
        done = 0.0;
        for (int b = 0; b < blk; ++b)
            done = done + tot[(size_t)b * n_m];
    }
    return done + S.part[((size_t)t * n_m + mi) * G.n_P + pi];
}

// Rows 2 and 9 of Table 1 are monotone in A = g(s) k for a fixed P (q >= 1,
// floor(log2 P) >= 1, rounding is monotone), so their minima over s are
//   min_s T2 = fma(q, min_s A, L),   min_s T9 = fma(fl, min_s A, cl L)
// exactly, and only min_s A (one v_min per (m, s)) is tracked in the sweeps.
// The segment size is then needed only in the cells that row 2 or 9 wins: there
// the candidates are walked once more, in ascending order, for the first s whose
// value equals the minimum (several A can round to the same time, so this is
// not simply the s of the smallest A).
//
// One lane per m, PC process counts per lane.  want[p]: 0 = nothing to find,
// else the row (2 or 9) that won cell p; V[p] its time.  cand(si, sd, rcp, gs)
// supplies the wave-uniform scalars of candidate si.  found[p] receives s.
template <int PC, class Cand>
__device__ __forceinline__ void first_s_of_flat_or_binomial(
    int n_cand, double limd, double md, double L, const double (&q)[PC], const double (&fl)[PC],
    const double (&clL)[PC], const int (&want)[PC], const double (&V)[PC], uint32_t (&found)[PC],
    Cand cand)
{
    bool open[PC];
#pragma unroll
    for (int p = 0; p < PC; ++p)
        open[p] = want[p] != 0;
    for (int si = 0; si < n_cand; ++si) {
        double sd, rcp_s, gs;
        cand(si, sd, rcp_s, gs);
        if (sd <= limd) {
            double A, B, C;
            segment_terms(md, sd, rcp_s, gs, L, A, B, C);
#pragma unroll
            for (int p = 0; p < PC; ++p) {
                const double Tv = want[p] == 2 ? __builtin_fma(q[p], A, L)
                                               : __builtin_fma(fl[p], A, clL[p]);
                if (open[p] && Tv == V[p]) {
                    found[p] = (uint32_t)sd;
                    open[p] = false;
                }
            }
        }
    }
}

// ---- sweep, few candidates: one lane per message size ------------------------
//
// A wave takes 64 consecutive m of one table and PC consecutive process counts.
// P and s are wave-uniform loop variables (their terms live in scalar
// registers); A, B are computed in the lane once per (m, s) and shared by the PC
// process counts.  Per (P, s) and segmented row: one fma, one compare, the
// running minimum and the index of the candidate that attained it (strict '<'
// in ascending s: ties go to the smallest s).

template <int PC>
__global__ void __launch_bounds__(256) k_sweep_m(DeviceTables T, DeviceGrid G, Scratch S,
                                                 plogp_cell_dev *out, int n_mg, int n_pcg)
{
    // the four waves of a workgroup share the table and the m group and take four
    // consecutive chunks of PC process counts; the per-candidate scalars (s, 1/s,
    // g(s)) are staged in LDS once for all of them
    __shared__ double sS[SWEEP_M_MAX_S], sR[SWEEP_M_MAX_S], sG[SWEEP_M_MAX_S];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    int bid = blockIdx.x;
    const int pcg = bid % n_pcg;
    bid /= n_pcg;
    const int mg = bid % n_mg;
    const int t = bid / n_mg;
    const int pc = pcg * 4 + wave;
    for (int si = threadIdx.x; si < G.n_s; si += blockDim.x) {
        sS[si] = (double)G.s[si];
        sR[si] = S.rcp[si];
        sG[si] = S.gs[(size_t)t * G.n_s + si];
    }
    __syncthreads();
    if (pc * PC >= G.n_P)
        return;

    const int mi = mg * 64 + lane;
    const bool active = mi < G.n_m;
    const u64 m = active ? G.m[mi] : 1;
    const double md = (double)m;
    const u64 lim = active ? (m < G.s_cap ? m : G.s_cap) : 0;
    const double limd = (double)lim;         // exact: at most m < 2^53 (0 for an idle lane)
    const double L = T.L[t];
    const uint32_t mask = G.mask;

    uint32_t Pv[PC];
    double q[PC], fl[PC], clL[PC];
#pragma unroll
    for (int p = 0; p < PC; ++p) {
        const int pi = pc * PC + p;
        Pv[p] = pi < G.n_P ? G.P[pi] : 2u;
        q[p] = (double)(Pv[p] - 1);
        fl[p] = (double)floor_log2(Pv[p]);
        clL[p] = (double)ceil_log2(Pv[p]) * L;
    }
    double b5[PC];
    int i5[PC];
#pragma unroll
    for (int p = 0; p < PC; ++p) {
        b5[p] = INFINITY;
        i5[p] = 0;
    }
    double amin = INFINITY;                  // min over s of A = g(s) k (rows 2 and 9)
    int n_seen = 0;                          // candidates walked (wave-uniform)
    if ((mask & 0x224u) && G.n_s > 0) {
        // the scalars of the next candidate are read from LDS while this one computes
        double sd_n = sS[0], rcp_n = sR[0], gs_n = sG[0];
        for (int si = 0; si < G.n_s; ++si) {
            const double sd = sd_n, rcp_s = rcp_n, gsv = gs_n;
            const int nx = si + 1 < G.n_s ? si + 1 : si;
            sd_n = sS[nx];
            rcp_n = sR[nx];
            gs_n = sG[nx];
            const bool valid = sd <= limd;
            if (__ballot(valid) == 0)
                break;                       // the candidates ascend: nothing further competes
            n_seen = si + 1;
            if (valid) {
                double A, B, C;
                segment_terms(md, sd, rcp_s, gsv, L, A, B, C);
                amin = min_f64(amin, A);
#pragma unroll
                for (int p = 0; p < PC; ++p) {
                    const double T5 = __builtin_fma(q[p], C, B);
                    i5[p] = T5 < b5[p] ? si : i5[p];
                    b5[p] = min_f64(b5[p], T5);
                }
            }
        }
    }
    if (!active)
        return;
    const size_t n_m = (size_t)G.n_m;
    const double gm = S.gm[(size_t)t * n_m + mi];
    const double g1 = S.g1[t];
    const size_t plane = n_m * G.n_P;

    // everything the PC cells read is fetched before the first of them is stored
    double s11[PC], s12[PC];
    uint32_t s5[PC];
    double done[PC];                         // finished blocks of the chain sum before each P
#pragma unroll
    for (int p = 0; p < PC; ++p)
        done[p] = 0.0;
    const size_t n_mu = (size_t)G.n_mu;      // the chain sums are kept per distinct size
    const int um = G.m_map[mi];
    if (mask & (1u << 11)) {
        const double *tot = S.blk + (size_t)t * G.n_blk * n_mu + um;
        if (G.blk_is_prefix) {
            const double *pre = S.pre + ((size_t)t * n_mu + um) * G.n_P;
#pragma unroll
            for (int p = 0; p < PC; ++p)
                done[p] = pre[pc * PC + p < G.n_P ? pc * PC + p : G.n_P - 1];
        } else {
            // few blocks (at most 32): the totals are added here, in ascending order; the
            // P of the chunk ascend, so one pass over the blocks serves all of them, and
            // the loads of eight blocks are in flight together
            int last = 0;
#pragma unroll
            for (int p = 0; p < PC; ++p) {
                const int blk = (int)((Pv[p] - 1u) / SUM_BLOCK);
                last = blk > last ? blk : last;
            }
            double acc = 0.0;
            for (int b0 = 0; b0 < last; b0 += 8) {
                double tv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    tv[u] = b0 + u < last ? tot[(size_t)(b0 + u) * n_mu] : 0.0;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (b0 + u < last) {
                        acc = acc + tv[u];
#pragma unroll
                        for (int p = 0; p < PC; ++p)
                            if ((int)((Pv[p] - 1u) / SUM_BLOCK) == b0 + u + 1)
                                done[p] = acc;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int p = 0; p < PC; ++p) {
        const int pi = pc * PC + p < G.n_P ? pc * PC + p : G.n_P - 1;
        s11[p] = s12[p] = 0.0;
        if (mask & (1u << 11))
            s11[p] = done[p] + S.part[((size_t)t * n_mu + um) * G.n_P + pi];
        if (mask & (1u << 12))
            s12[p] = S.sum2[((size_t)t * n_m + mi) * (G.cl_max + 1) + ceil_log2(Pv[p])];
        s5[p] = b5[p] < INFINITY ? (uint32_t)sS[i5[p]] : 0u;
    }
    Best bc[PC];
    if (mask & 0x3FFu) {
        int want[PC];
        double V[PC];
        uint32_t found[PC];
        bool any = false;
#pragma unroll
        for (int p = 0; p < PC; ++p) {
            const double t2 = amin < INFINITY ? __builtin_fma(q[p], amin, L) : INFINITY;
            const double t9 = amin < INFINITY ? __builtin_fma(fl[p], amin, clL[p]) : INFINITY;
            bc[p] = decide_bcast(mask, q[p], fl[p], (double)ceil_log2(Pv[p]), gm, L, g1, t2, 0u,
                                 b5[p], s5[p], t9, 0u);
            want[p] = (bc[p].id == 2u || bc[p].id == 9u) ? (int)bc[p].id : 0;
            V[p] = bc[p].t;
            found[p] = 0u;
            any = any || want[p] != 0;
        }
        if (__ballot(any) != 0) {
            first_s_of_flat_or_binomial<PC>(
                n_seen, limd, md, L, q, fl, clL, want, V, found,
                [&](int si, double &sd, double &rcp_s, double &g) {
                    sd = sS[si];
                    rcp_s = sR[si];
                    g = sG[si];
                });
#pragma unroll
            for (int p = 0; p < PC; ++p)
                if (want[p] != 0)
                    bc[p].s = found[p];
        }
    }
#pragma unroll
    for (int p = 0; p < PC; ++p) {
        const int pi = pc * PC + p;
        if (pi >= G.n_P)
            break;
        plogp_cell_dev *o = out + (size_t)t * G.n_ops * plane + (size_t)mi * G.n_P + pi;
        const double cl = (double)ceil_log2(Pv[p]);
        if (mask & 0x3FFu) {
            store_cell(o, bc[p]);
            o += plane;
        }
        if (mask & 0x1C00u)
            store_cell(o, decide_scatter(mask, q[p], cl, gm, L, s11[p], s12[p]));
    }
}

// ---- sweep, many candidates: one lane per segment size -----------------------

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_move(double v)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(lo, lo, CTRL, ROW_MASK, 0xf, false);
    hi = __builtin_amdgcn_update_dpp(hi, hi, CTRL, ROW_MASK, 0xf, false);
    return __hiloint2double(hi, lo);
}

// Minimum over the 64 lanes of a fully active wave, returned in every lane.
// DPP butterflies inside each row of 16 lanes (quad permutes, half-row and row
// mirrors), then the row broadcasts 15 and 31 fold the four rows into lane 63.
__device__ __forceinline__ double wave_min(double v)
{
    v = min_f64(v, dpp_move<0xB1, 0xf>(v));            // quad_perm [1,0,3,2]
    v = min_f64(v, dpp_move<0x4E, 0xf>(v));            // quad_perm [2,3,0,1]
    v = min_f64(v, dpp_move<0x141, 0xf>(v));           // row_half_mirror
    v = min_f64(v, dpp_move<0x140, 0xf>(v));           // row_mirror
    v = min_f64(v, dpp_move<0x142, 0xa>(v));           // row_bcast:15 into rows 1, 3
    v = min_f64(v, dpp_move<0x143, 0xc>(v));           // row_bcast:31 into rows 2, 3
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 63);
    return __hiloint2double(hi, lo);
}

// ---- sweep, few candidates, many process counts: one lane per P -----------------
//
// A wave takes 64 consecutive process counts of the grid (its lanes) and walks
// over message sizes.  Everything that depends on (m, s) only -- A, B (from
// k_terms), C, the candidate count, g(m) -- is the same in all lanes then: per
// candidate the lanes do one fma, one compare, the index select and the running
// minimum for row 5 of Table 1; min_s A for rows 2 and 9 is one reduction over the
// wave per m.  A cell costs two coalesced 16-byte stores.  The sizes of a wave lie
// n_w apart, so every wave meets the same mix of short and long candidate lists;
// the loads for the next size are issued before the current one is worked on.
// NSV: candidates per lane when a row of (m, s) terms is moved (n_s <= 64 NSV).
template <int NSV, bool ALL, int PPL>
__global__ void __launch_bounds__(256) k_sweep_p(DeviceTables T, DeviceGrid G, Scratch S,
                                                 plogp_cell_dev *out, int t0, int n_w)
{
    // the loops below read up to 7 entries past the last candidate: rows are 8 longer
    constexpr int ROW = 64 * NSV + 8;
    __shared__ double sC[ROW];                       // g(s) + L (0 past the end)
    __shared__ uint32_t sSv[ROW];                    // s
    __shared__ double rowB[4][ROW];                  // B of the current size (+inf past the end)
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // grid: x = group of four waves, y = group of 64 PPL process counts, z = table (from t0)
    const int wq = (int)blockIdx.x, pg = (int)blockIdx.y, t = t0 + (int)blockIdx.z;
    const int w = wq * 4 + wave;
    const bool has_work = w < n_w && w < G.n_m;
    const uint32_t mask = ALL ? 0x1FFFu : G.mask;      // ALL: every strategy competes
    const int n_P = G.n_P, n_s = G.n_s, n_blk = G.n_blk;
    const size_t n_m = (size_t)G.n_m;
    const double L = T.L[t];
    const double g1 = S.g1[t];
    const bool chain = (mask & (1u << 11)) != 0, binom = (mask & (1u << 12)) != 0;
    const bool seg = (mask & 0x224u) != 0 && n_s > 0;
    const size_t plane = n_m * n_P;
    // a lane takes PPL process counts, 64 apart (so that every store of a wave is one run)
    int pi[PPL], cli[PPL], blk[PPL], bmin[PPL], bmax[PPL];
    bool active[PPL];
    double q[PPL], fl[PPL], cl[PPL], clL[PPL];
#pragma unroll
    for (int h = 0; h < PPL; ++h) {
        const int base = (pg * PPL + h) * 64;
        pi[h] = base + lane;
        active[h] = pi[h] < n_P;
        const uint32_t Pv = G.P[active[h] ? pi[h] : n_P - 1];
        q[h] = (double)(Pv - 1u);
        cli[h] = ceil_log2(Pv);
        fl[h] = (double)floor_log2(Pv);
        cl[h] = (double)cli[h];
        clL[h] = cl[h] * L;
        blk[h] = (int)((Pv - 1u) / SUM_BLOCK);
        // the smallest and the largest block index among the lanes (the P of the grid ascend;
        // an empty half repeats the last P of the grid)
        const int here = n_P - base < 64 ? n_P - base : 64;
        bmin[h] = __builtin_amdgcn_readfirstlane(blk[h]);
        bmax[h] = __builtin_amdgcn_readlane(blk[h], here > 0 ? here - 1 : 0);
    }
    plogp_cell_dev *const obase = out + (size_t)t * G.n_ops * plane + pi[0];

    // what is fetched one size ahead
    double fB[NSV], f_part[PPL], f_s12[PPL], f_done[PPL], f_gm, f_amin = INFINITY;
    int f_nv;
#pragma unroll
    for (int h = 0; h < PPL; ++h)
        f_part[h] = f_s12[h] = f_done[h] = 0.0;
    // row of the chain sums (kept per distinct size) of the size fetched next: read one size
    // earlier still, so that the fetch does not wait for it
    int um_next = chain && has_work ? G.m_map[w] : 0;
    // the sizes of a wave lie n_w apart: the rows of the per-size arrays are reached by adding
    // a stride to running pointers (no multiplications per size); the chain sums are kept per
    // distinct size and go through the row map
    const double *p_gm = S.gm + (size_t)t * n_m + w;
    const double *p_amin = S.amin + (size_t)t * n_m + w;
    const int *p_nv = S.nv + w;
    const double *p_B = S.segB + ((size_t)t * n_m + w) * n_s + lane;
    const double *p_s12 = S.sum2 + ((size_t)t * n_m + w) * (G.cl_max + 1);
    const size_t stride_B = (size_t)n_w * n_s, stride_s12 = (size_t)n_w * (G.cl_max + 1);
    const double *const part_t = S.part + (size_t)t * G.n_mu * n_P;
    const double *const pre_t = S.pre + (size_t)t * G.n_mu * n_P;
    const double *const blk_t = S.blk + ((size_t)t * n_blk + lane) * G.n_mu;
    auto fetch = [&](int mi) {
        f_gm = *p_gm;
        f_nv = *p_nv;
        p_gm += n_w;
        p_nv += n_w;
        if (seg) {
            f_amin = *p_amin;
            p_amin += n_w;
#pragma unroll
            for (int k = 0; k < NSV; ++k)
                fB[k] = lane + 64 * k < n_s ? p_B[64 * k] : INFINITY;
            p_B += stride_B;
        }
        if (chain) {
            const uint32_t um = (uint32_t)um_next;
            um_next = G.m_map[mi + n_w < (int)n_m ? mi + n_w : mi];
            const double *row = part_t + (u64)um * (uint32_t)n_P;
#pragma unroll
            for (int h = 0; h < PPL; ++h)
                f_part[h] = row[active[h] ? pi[h] : n_P - 1];
            if (G.blk_is_prefix) {
                const double *prow = pre_t + (u64)um * (uint32_t)n_P;
#pragma unroll
                for (int h = 0; h < PPL; ++h)
                    f_done[h] = prow[active[h] ? pi[h] : n_P - 1];
            } else {                   // few blocks: lane b holds the total of block b
                f_done[0] = lane < n_blk - 1 ? blk_t[um] : 0.0;
            }
        }
        if (binom) {
#pragma unroll
            for (int h = 0; h < PPL; ++h)
                f_s12[h] = p_s12[cli[h]];
            p_s12 += stride_s12;
        }
    };
    // the first size's inputs are on their way while the candidates go to LDS
    if (has_work)
        fetch(w);
    for (int si = threadIdx.x; si < ROW; si += blockDim.x) {
        sC[si] = si < G.n_s ? S.segC[(size_t)t * G.n_s + si] : 0.0;
        sSv[si] = si < G.n_s ? (uint32_t)G.s[si] : 0u;
        if (si >= 64 * NSV) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                rowB[k][si] = INFINITY;
        }
    }
    __syncthreads();
    if (!has_work)
        return;
    for (int mi = w; mi < (int)n_m; mi += n_w) {
        const double gm = f_gm;
        double part[PPL], s12[PPL], dn[PPL];
#pragma unroll
        for (int h = 0; h < PPL; ++h) {
            part[h] = f_part[h];
            s12[h] = f_s12[h];
            dn[h] = f_done[h];
        }
        const int nv = f_nv;
        const double amin = f_amin;      // min over s of A = g(s) k, from k_terms
        const size_t row_now = (size_t)t * n_m + mi;
        if (seg) {
#pragma unroll
            for (int k = 0; k < NSV; ++k)
                rowB[wave][lane + 64 * k] = fB[k];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (mi + n_w < (int)n_m)
            fetch(mi + n_w);

        // row 5: min over s of fma(q, C, B).  The loop keeps the minimum and in which batch of
        // eight candidates it first appeared; the candidate itself is looked for afterwards,
        // and only where row 5 wins the cell.
        double b5[PPL];
        int i5[PPL];
#pragma unroll
        for (int h = 0; h < PPL; ++h) {
            b5[h] = INFINITY;
            i5[h] = 0;
        }
        if (mask & 0x20u) {
            // eight candidates per round trip to LDS; past the last competing one B is
            // +inf (and C is finite), so the value is +inf and never taken
            for (int s0 = 0; s0 < nv; s0 += 8) {
                double Bv[8], Cv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    Bv[u] = rowB[wave][s0 + u];
                    Cv[u] = sC[s0 + u];
                }
#pragma unroll
                for (int h = 0; h < PPL; ++h) {
                    double cur = INFINITY;
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        cur = min_f64(cur, __builtin_fma(q[h], Cv[u], Bv[u]));
                    i5[h] = cur < b5[h] ? s0 : i5[h];
                    b5[h] = min_f64(b5[h], cur);
                }
            }
        }

        plogp_cell_dev *o = obase + (size_t)mi * n_P;
        if (mask & 0x3FFu) {
#pragma unroll
            for (int h = 0; h < PPL; ++h) {
                const double t2 = amin < INFINITY ? __builtin_fma(q[h], amin, L) : INFINITY;
                const double t9 = amin < INFINITY ? __builtin_fma(fl[h], amin, clL[h]) : INFINITY;
                Best bc = decide_bcast(mask, q[h], fl[h], cl[h], gm, L, g1, t2, 0u, b5[h], 0u, t9, 0u);
                // a winning row 5: the first candidate of the remembered batch that attains the
                // minimum (lanes differ in their batch: per-lane LDS reads of its eight candidates)
                if (__ballot(active[h] && bc.id == 5u) != 0) {
                    double Bv[8], Cv[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        Bv[u] = rowB[wave][i5[h] + u];
                        Cv[u] = sC[i5[h] + u];
                    }
                    int at5 = i5[h];
#pragma unroll
                    for (int u = 7; u >= 0; --u)        // descending: the first match stays
                        at5 = __builtin_fma(q[h], Cv[u], Bv[u]) == b5[h] ? i5[h] + u : at5;
                    const uint32_t s_at = sSv[at5];
                    bc.s = bc.id == 5u ? s_at : bc.s;
                }
                // a winning row 2 or 9: the first candidate whose value equals the minimum
                bool open = active[h] && (bc.id == 2u || bc.id == 9u);
                if (__ballot(open) != 0) {
                    const double mul = bc.id == 2u ? q[h] : fl[h], add = bc.id == 2u ? L : clL[h];
                    uint32_t found = 0u;
                    for (int s0 = 0; s0 < nv; s0 += 4) {     // past the last candidate A is +inf
                        double Av[4];
                        uint32_t Sv[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            Av[u] = s0 + u < n_s ? S.segA[row_now * n_s + s0 + u] : INFINITY;
                            Sv[u] = sSv[s0 + u];
                        }
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const bool hit = open && __builtin_fma(mul, Av[u], add) == bc.t;
                            found = hit ? Sv[u] : found;
                            open = open && !hit;
                        }
                        if (__ballot(open) == 0)
                            break;
                    }
                    if (bc.id == 2u || bc.id == 9u)
                        bc.s = found;
                }
                if (active[h])
                    store_cell(o + 64 * h, bc);
            }
            o += plane;
        }
        if (mask & 0x1C00u) {
            double s11[PPL];
#pragma unroll
            for (int h = 0; h < PPL; ++h)
                s11[h] = 0.0;
            if (chain) {
                double done[PPL];
                if (!G.blk_is_prefix) {
                    // the finished blocks are added in ascending order, the same sum in every
                    // lane; a lane keeps, per process count, the value that belongs to its block
                    const double tot = dn[0];
                    double acc = 0.0;
                    for (int b = 0; b < bmin[0]; ++b)
                        acc = acc + __hiloint2double(
                                        __builtin_amdgcn_readlane(__double2hiint(tot), b),
                                        __builtin_amdgcn_readlane(__double2loint(tot), b));
#pragma unroll
                    for (int h = 0; h < PPL; ++h)
                        done[h] = acc;               // lanes of block bmin[0]
                    for (int b = bmin[0]; b < bmax[PPL - 1]; ++b) {
                        acc = acc + __hiloint2double(
                                        __builtin_amdgcn_readlane(__double2hiint(tot), b),
                                        __builtin_amdgcn_readlane(__double2loint(tot), b));
#pragma unroll
                        for (int h = 0; h < PPL; ++h)
                            done[h] = blk[h] == b + 1 ? acc : done[h];
                    }
                } else {
#pragma unroll
                    for (int h = 0; h < PPL; ++h)
                        done[h] = dn[h];
                }
#pragma unroll
                for (int h = 0; h < PPL; ++h)
                    s11[h] = done[h] + part[h];
            }
#pragma unroll
            for (int h = 0; h < PPL; ++h)
                if (active[h])
                    store_cell(o + 64 * h, decide_scatter(mask, q[h], cl[h], gm, L, s11[h], s12[h]));
        }
        __builtin_amdgcn_wave_barrier();
    }
}

constexpr int SWEEP_S_CHUNK = 1024;     // candidates staged in LDS per pass (16 per lane)
constexpr int SWEEP_S_MAX_WAVES = 8;
constexpr int SWEEP_S_PASSES = 64;      // passes whose minimum of A is remembered

// A workgroup takes one (table, m) and up to SWEEP_S_MAX_WAVES groups of GP
// process counts, one group per wave; lanes run over the candidates s.  A, B, C
// of a pass of SWEEP_S_CHUNK candidates are computed once by the whole
// workgroup into LDS (double-buffered) and read by every wave.  In the loop a
// wave keeps, per process count, the running minimum of the segmented chain
// (row 5: one fma and one min per value); per lane it remembers in which pass
// each row-5 minimum first appeared.  The minimum of A (rows 2 and 9 are monotone
// in A, and A does not depend on P) is formed once per pass, by wave 0, from the
// minima that the threads filling the pass leave in LDS.  At the end the row-5
// minima are reduced across lanes, the winner is chosen in id order, and only for a
// winning segmented row the smallest s that attains the minimum is looked for:
// for row 5 among the candidates of the pass the holding lanes remember, for
// rows 2 and 9 by one ascending walk over the candidates.
template <int GP>
__global__ void __launch_bounds__(64 * SWEEP_S_MAX_WAVES)
k_sweep_s(DeviceTables T, DeviceGrid G, Scratch S, plogp_cell_dev *out, int n_ptiles)
{
    __shared__ double2 AB[2][SWEEP_S_CHUNK];           // {B, C} of the candidates of a pass
    __shared__ double Cs[2][SWEEP_S_CHUNK];            // (only the reduction at the end uses it)
    __shared__ double passMinA[SWEEP_S_PASSES];        // min of A over each of the first passes
    __shared__ double fillMinA[2][64 * SWEEP_S_MAX_WAVES];   // per filling thread: min of A over its candidates
    __shared__ double allMinA;                         // min of A over every candidate

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n_waves = blockDim.x >> 6;
    int bid = blockIdx.x;
    const int ptile = bid % n_ptiles;
    bid /= n_ptiles;
    const int mi = bid % G.n_m;
    const int t = bid / G.n_m;
    const int p0 = (ptile * n_waves + wave) * GP;      // first P index of this wave
    const bool has_work = p0 < G.n_P;

    const u64 m = G.m[mi];
    const double md = (double)m;
    const double L = T.L[t];
    const uint32_t mask = G.mask;
    const double *gs = S.gs + (size_t)t * G.n_s;

    const int nv = S.nv[mi];                           // candidates s <= min(m, s_cap)
    const int n_chunks = (nv + SWEEP_S_CHUNK - 1) / SWEEP_S_CHUNK;

    double q[GP];                                      // wave-uniform: kept in scalar registers
#pragma unroll
    for (int p = 0; p < GP; ++p) {
        const uint32_t Pv = (p0 + p < G.n_P) ? G.P[p0 + p] : 2u;
        const double qv = (double)(Pv - 1);
        q[p] = __hiloint2double(__builtin_amdgcn_readfirstlane(__double2hiint(qv)),
                                __builtin_amdgcn_readfirstlane(__double2loint(qv)));
    }
    double best5[GP];
    int blk5[GP];
#pragma unroll
    for (int p = 0; p < GP; ++p) {
        best5[p] = INFINITY;
        blk5[p] = 0;
    }
    double amin = INFINITY;                            // (wave 0 only, the same in its lanes)
    // What lane p < GP needs at the end to decide its cells is asked for now, so that the end
    // of the wave does not wait for device memory: its process count, g(m), g(1), the two
    // Scatter sums.
    const int pi = p0 + lane;
    const bool mine = lane < GP && pi < G.n_P;
    uint32_t Pv = 2u;
    double gm = 0.0, g1 = 0.0, s11 = 0.0, s12 = 0.0;
    if (has_work) {
        Pv = G.P[mine ? pi : G.n_P - 1];
        gm = S.gm[(size_t)t * G.n_m + mi];
        g1 = S.g1[t];
        if (mine && (mask & (1u << 11)))
            s11 = chain_sum_of(G, S, t, mi, pi, Pv);
        if (mine && (mask & (1u << 12)))
            s12 = S.sum2[((size_t)t * G.n_m + mi) * (size_t)(G.cl_max + 1) + ceil_log2(Pv)];
    }

    // Filling a pass: the loads of the per-candidate scalars are issued before the
    // previous pass is consumed, the arithmetic and the LDS stores come after it.
    // A workgroup has at least SWEEP_S_CHUNK / FILL_SLOTS threads.
    constexpr int FILL_SLOTS = 2;
    double f_s[FILL_SLOTS], f_rcp[FILL_SLOTS], f_gs[FILL_SLOTS];
    auto fill_load = [&](int c) {
#pragma unroll
        for (int k = 0; k < FILL_SLOTS; ++k) {
            const int si = c * SWEEP_S_CHUNK + (int)threadIdx.x + k * (int)blockDim.x;
            const int idx = si < nv ? si : nv - 1;
            f_s[k] = (double)G.s[idx];
            f_rcp[k] = S.rcp[idx];
            f_gs[k] = gs[idx];
        }
    };
    auto fill_store = [&](int c) {
        const int buf = c & 1;
        double mine_A = INFINITY;
#pragma unroll
        for (int k = 0; k < FILL_SLOTS; ++k) {
            const int e = (int)threadIdx.x + k * (int)blockDim.x;
            if (e < SWEEP_S_CHUNK) {
                double A = INFINITY, B = INFINITY, C = 0.0;
                if (c * SWEEP_S_CHUNK + e < nv)
                    segment_terms(md, f_s[k], f_rcp[k], f_gs[k], L, A, B, C);
                AB[buf][e] = make_double2(B, C);           // one 16-byte read per candidate in the loop
                mine_A = min_f64(mine_A, A);
            }
        }
        // A does not depend on the process count: its minimum over a pass is formed from these
        // per-thread minima by one wave, not by every wave over every candidate
        fillMinA[buf][threadIdx.x] = mine_A;
    };
    if (n_chunks > 0) {
        fill_load(0);
        fill_store(0);
    }
    __syncthreads();
    for (int c = 0; c < n_chunks; ++c) {
        if (c + 1 < n_chunks)
            fill_load(c + 1);
        if (has_work) {
            const int buf = c & 1;
            const int len = min(SWEEP_S_CHUNK, nv - c * SWEEP_S_CHUNK);
            const int steps = (len + 63) >> 6;
            double cur5[GP];
#pragma unroll
            for (int p = 0; p < GP; ++p)
                cur5[p] = INFINITY;
#pragma unroll 2
            for (int i = 0; i < steps; ++i) {
                const double2 bc = AB[buf][64 * i + lane];
#pragma unroll
                for (int p = 0; p < GP; ++p)
                    cur5[p] = min_f64(cur5[p], __builtin_fma(q[p], bc.y, bc.x));
            }
#pragma unroll
            for (int p = 0; p < GP; ++p) {
                blk5[p] = cur5[p] < best5[p] ? c : blk5[p];
                best5[p] = min_f64(best5[p], cur5[p]);
            }
            if (wave == 0) {                           // wave 0 always has work
                double curA = INFINITY;
                for (int k = lane; k < (int)blockDim.x; k += 64)
                    curA = min_f64(curA, fillMinA[buf][k]);
                const double pm = wave_min(curA);
                amin = min_f64(amin, pm);
                if (lane == 0 && c < SWEEP_S_PASSES)
                    passMinA[c] = pm;
                if (lane == 0 && c + 1 == n_chunks)
                    allMinA = amin;
            }
        }
        if (c + 1 < n_chunks)
            fill_store(c + 1);
        __syncthreads();
    }
    if (!has_work)
        return;

    // The minimum of row 5 over the lanes, for all process counts of the group at once: the
    // lanes leave their minima in LDS (the candidate buffers are free now, every wave has
    // passed the last barrier), lane p reads the 64 minima of process count p0 + p (the
    // columns are 65 apart where they fit, so that the lanes hit different banks) and keeps
    // their minimum.
    const double Aw = (mask & 0x204u) && n_chunks > 0 ? allMinA : INFINITY;
    const bool haveA = Aw < INFINITY;
    double V5 = INFINITY;
    if (mask & (1u << 5)) {
        static_assert(GP <= 12, "columns of the reduction buffer");
        // per wave 512 doubles of AB and 256 of Cs: 7 + 3 padded columns, or 8 + 4 plain ones
        constexpr int LD = GP <= 10 ? 65 : 64, NLO = GP <= 10 ? 7 : 8;
        double *lo = reinterpret_cast<double *>(&AB[0][0]) + wave * 512;
        double *hi = &Cs[0][0] + wave * 256;
#pragma unroll
        for (int p = 0; p < GP; ++p)
            (p < NLO ? lo + LD * p : hi + LD * (p - NLO))[lane] = best5[p];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        // in two steps, so that most lanes take part: lane l takes a stretch of the 64 minima of
        // process count l % GP, then lane p the results of its stretches
        constexpr int NPART = 64 / GP, PER = (64 + NPART - 1) / NPART;
        double *mid = &fillMinA[0][0] + wave * 64;     // (free: every wave is past the last pass)
        if (lane < GP * NPART) {
            const int pp = lane % GP, part = lane / GP;
            const double *col = pp < NLO ? lo + LD * pp : hi + LD * (pp - NLO);
            double v[PER];
#pragma unroll
            for (int u = 0; u < PER; ++u)
                v[u] = col[part * PER + u < 64 ? part * PER + u : 63];
            double least = v[0];
#pragma unroll
            for (int u = 1; u < PER; ++u)
                least = min_f64(least, v[u]);
            mid[lane] = least;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (lane < GP) {
#pragma unroll
            for (int part = 0; part < NPART; ++part)
                V5 = min_f64(V5, mid[part * GP + lane]);
        }
    }

    // lanes 0..GP-1 decide one Broadcast cell each: the segmented rows' minima, the
    // unsegmented rows, arg-min.  The segment size is looked for afterwards, and only in
    // the cells that a segmented row wins.
    const double qv = (double)(Pv - 1);
    const int fli = floor_log2(Pv), cli = ceil_log2(Pv);
    const size_t plane = (size_t)G.n_m * G.n_P;
    plogp_cell_dev *o = out + (size_t)t * G.n_ops * plane + (size_t)mi * G.n_P + (mine ? pi : 0);
    Best bc = {INFINITY, 0u, 0xFFFFFFFFu};
    if (mask & 0x3FFu) {
        const double t2 = ((mask & (1u << 2)) && haveA) ? __builtin_fma(qv, Aw, L) : INFINITY;
        const double t9 = ((mask & (1u << 9)) && haveA)
                              ? __builtin_fma((double)fli, Aw, (double)cli * L) : INFINITY;
        bc = decide_bcast(mask, qv, (double)fli, (double)cli, gm, L, g1, t2, 0u, V5, 0u, t9, 0u);
        const unsigned long long need =
            __ballot(mine && (bc.id == 2u || bc.id == 5u || bc.id == 9u));
        if (need != 0) {
            // Row 5: every lane that holds the minimum V of process count p names the pass it
            // first saw it in; that lane's 16 candidates of the pass are evaluated again, by 16
            // lanes, and the first that gives V is its earliest.  Four such (process count,
            // holding lane) queries are worked on at once, one per quarter of the wave; lane p
            // keeps the smallest index found for process count p and the candidate there.
            int first_v = 0x7FFFFFFF;
            double s_v = 0.0;
            int qc = 0, ql = 0, qp = 0;                    // the query of this lane's quarter
            double qV = 0.0, qq = 0.0;
            int nq = 0;                                    // queries waiting (wave-uniform)
            auto from_lane = [&](double v, int l) {
                return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), l),
                                        __builtin_amdgcn_readlane(__double2loint(v), l));
            };
            auto flush = [&]() {
                const bool live = (lane >> 4) < nq;
                const int si = qc * SWEEP_S_CHUNK + 64 * (lane & 15) + ql;
                const int idx = si < nv ? si : nv - 1;
                const double r_s = (double)G.s[idx];
                double A, B, C;
                segment_terms(md, r_s, S.rcp[idx], gs[idx], L, A, B, C);
                const bool hit = live && si < nv && __builtin_fma(qq, C, B) == qV;
                const unsigned long long hits = __ballot(hit);
                for (int j = 0; j < nq; ++j) {
                    const unsigned h = (unsigned)(hits >> (16 * j)) & 0xFFFFu;
                    if (h == 0u)
                        continue;
                    const int k = __builtin_ctz(h);
                    const int cand = __builtin_amdgcn_readlane(qc, 16 * j) * SWEEP_S_CHUNK + 64 * k +
                                     __builtin_amdgcn_readlane(ql, 16 * j);
                    const double s_c = from_lane(r_s, 16 * j + k);
                    if (lane == __builtin_amdgcn_readlane(qp, 16 * j) && cand < first_v) {
                        first_v = cand;
                        s_v = s_c;
                    }
                }
                nq = 0;
            };
            auto push = [&](int p, int l, int c, double V, double q_p) {
                const bool slot = (lane >> 4) == nq;
                qc = slot ? c : qc;
                ql = slot ? l : ql;
                qp = slot ? p : qp;
                qV = slot ? V : qV;
                qq = slot ? q_p : qq;
                if (++nq == 4)
                    flush();
            };
#pragma unroll
            for (int p = 0; p < GP; ++p) {
                if (!((need >> p) & 1ull) || __builtin_amdgcn_readlane((int)bc.id, p) != 5)
                    continue;                              // wave-uniform
                const double V = from_lane(bc.t, p);
                unsigned long long holders = __ballot(best5[p] == V);
                while (holders != 0) {                     // more than one lane only on exact ties
                    const int l = __builtin_ctzll(holders);
                    holders &= holders - 1;
                    push(p, l, __builtin_amdgcn_readlane(blk5[p], l), V, q[p]);
                }
            }
            if (nq > 0)
                flush();
            if (bc.id == 5u)
                bc.s = first_v < nv ? (uint32_t)s_v : 0u;

            // Rows 2 and 9: the first pass whose minimum of A already gives V holds the
            // smallest such s; walk that pass in ascending order, 64 candidates at a time
#pragma unroll
            for (int p = 0; p < GP; ++p) {
                if (!((need >> p) & 1ull))
                    continue;                              // wave-uniform
                const int id = __builtin_amdgcn_readlane((int)bc.id, p);
                if (id == 5)
                    continue;
                const double V = from_lane(bc.t, p);
                int first = 0x7FFFFFFF;
                double s_first = 0.0;                      // the candidate at index `first`
                const uint32_t Pp = G.P[p0 + p];
                const double flp = (double)floor_log2(Pp);
                const double clLp = (double)ceil_log2(Pp) * L;
                const double mul = id == 2 ? q[p] : flp;
                const double add = id == 2 ? L : clLp;
                int c0 = 0;
                const int known = n_chunks < SWEEP_S_PASSES ? n_chunks : SWEEP_S_PASSES;
                while (c0 < known && __builtin_fma(mul, passMinA[c0], add) != V)
                    ++c0;
                for (int base = c0 * SWEEP_S_CHUNK; base < nv && first == 0x7FFFFFFF; base += 256) {
                    // four groups of 64 candidates per round trip to memory
                    double sdv[4], rcv[4], gsv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int si = base + 64 * u + lane;
                        const int idx = si < nv ? si : nv - 1;
                        sdv[u] = (double)G.s[idx];
                        rcv[u] = S.rcp[idx];
                        gsv[u] = gs[idx];
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        double A, B, C;
                        segment_terms(md, sdv[u], rcv[u], gsv[u], L, A, B, C);
                        const bool hit = base + 64 * u + lane < nv && __builtin_fma(mul, A, add) == V;
                        const unsigned long long hits = __ballot(hit);
                        if (hits != 0 && first == 0x7FFFFFFF) {
                            first = base + 64 * u + __builtin_ctzll(hits);
                            s_first = from_lane(sdv[u], __builtin_ctzll(hits));
                        }
                    }
                }
                if (lane == p)
                    bc.s = first < nv ? (uint32_t)s_first : 0u;
            }
        }
        if (mine)
            store_cell(o, bc);
        o += plane;
    }
    if (!mine)
        return;
    if (mask & 0x1C00u)
        store_cell(o, decide_scatter(mask, qv, (double)cli, gm, L, s11, s12));
}

// ---- whole path in one kernel, for batches of many tables -----------------
//
// One workgroup per (table, 256 message sizes), one lane per m, everything of
// that (table, m) row in the lane: g(m), the segment terms, the Scatter-chain sum walked along j while P ascends (the sum
// for a P is ready exactly when its cells are written), the binomial sum grown
// term by term with ceil(log2 P).  P and s are wave-uniform loops; P goes in
// chunks of FUSED_PC so that A and B are formed once per (m, s, chunk).  The
// cells of a chunk are transposed through LDS so that a store instruction writes
// 64-byte runs instead of 64 separate records.  No scratch in global memory:
// the only HBM traffic is the tables in and the decision table out.  Used when
// there are enough (table, m) rows to fill the chip, at most FUSED_NS candidates
// and few blocks of the chain sum.
constexpr int FUSED_NS = 24;
constexpr int FUSED_PC = 4;

// X[0] = 0 (virtual interval below the first sample, gap y_0, slope 0),
// X[1..n] = samples, X[n+1] = X[n+2] = +inf; YS[i] = {gap, slope} of interval i.
__device__ __forceinline__ int lds_interval(const double *X, int n, double z)
{
    return last_not_above(X + 1, n, z) + (z >= X[1] ? 1 : 0);
}

__device__ __forceinline__ double lds_gap(const double *X, const double2 *YS, int n, double z)
{
    const int i = lds_interval(X, n, z);
    const double2 ys = YS[i];
    return __builtin_fma(ys.y, z - X[i], ys.x);
}

__global__ void __launch_bounds__(256) k_fused(DeviceTables T, DeviceGrid G, plogp_cell_dev *out,
                                               int n_mchunks)
{
    extern __shared__ __align__(16) double fused_lds[];
    __shared__ double sS[FUSED_NS], sG[FUSED_NS], sR[FUSED_NS];
    __shared__ double sG1;
    // per wave and plane: 64 rows x FUSED_PC cells, rows padded by one cell
    __shared__ uint4 stage[4][2][64 * (FUSED_PC + 1)];

    const int t = blockIdx.x / n_mchunks, mc = blockIdx.x % n_mchunks;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n = T.n;
    double2 *YS = reinterpret_cast<double2 *>(fused_lds);      // n + 2 entries
    double *X = fused_lds + 2 * (n + 2);                       // n + 3 entries
    const double L = T.L[t];
    {
        const double *gx = T.x + (size_t)t * n, *gy = T.y + (size_t)t * n;
        for (int i = threadIdx.x; i < n; i += blockDim.x) {
            X[i + 1] = gx[i];
            YS[i + 1] = make_double2(gy[i], interval_slope(gx, gy, n, i));
        }
        if (threadIdx.x == 0) {
            X[0] = 0.0;
            X[n + 1] = INFINITY;
            X[n + 2] = INFINITY;
            YS[0] = make_double2(gy[0], 0.0);
            YS[n + 1] = make_double2(0.0, 0.0);
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < G.n_s) {
        const double sd = (double)G.s[threadIdx.x];
        const double g = lds_gap(X, YS, n, sd);
        sS[threadIdx.x] = sd;
        sG[threadIdx.x] = g;
        sR[threadIdx.x] = 1.0 / sd;
    }
    if (threadIdx.x == 0)
        sG1 = lds_gap(X, YS, n, 1.0);
    __syncthreads();

    const int mi = mc * blockDim.x + threadIdx.x;
    const bool active = mi < G.n_m;
    const u64 m = G.m[active ? mi : 0];
    const double md = (double)m;
    const u64 lim = active ? (m < G.s_cap ? m : G.s_cap) : 0;
    const double limd = (double)lim;       // exact: at most m < 2^53 (0 for an idle lane)
    const uint32_t mask = G.mask;
    const double g1 = sG1;
    const double gm = lds_gap(X, YS, n, md);

    // candidates that compete for some lane of the wave (they ascend), and the
    // minimum over s of A = g(s) k for this m (rows 2 and 9 are monotone in A)
    int wave_nv = 0;
    double amin = INFINITY;
    for (int si = 0; si < G.n_s; ++si) {
        const double sd = sS[si];
        const bool valid = sd <= limd;
        if (__ballot(valid) == 0)
            break;
        wave_nv = si + 1;
        if (valid && (mask & 0x204u)) {
            double A, B, C;
            segment_terms(md, sd, sR[si], sG[si], L, A, B, C);
            amin = min_f64(amin, A);
        }
    }

    // Scatter-chain walk.  Current interval: d = z - start, w = width, {yi, sl};
    // the next interval's end and {gap, slope} are fetched one crossing ahead.
    int iv = lds_interval(X, n, md);
    double xb = X[iv + 1];
    double d = md - X[iv], w = xb - X[iv];
    double yi = YS[iv].x, sl = YS[iv].y;
    double nxb = X[iv + 2];
    double2 nys = YS[iv + 1];
    double run = 0.0, done = 0.0;
    int j_done = 0;
    double s12 = 0.0;                      // Scatter-binomial sum, grown with ceil(log2 P)
    int cl_done = 0;

    const size_t plane = (size_t)G.n_m * G.n_P;
    plogp_cell_dev *o_tab = out + (size_t)t * G.n_ops * plane;
    const bool want_chain = (mask & (1u << 11)) != 0, want_binom = (mask & (1u << 12)) != 0;
    const bool has_b = (mask & 0x3FFu) != 0, has_s = (mask & 0x1C00u) != 0;
    const int row0 = mc * (int)blockDim.x + wave * 64;         // first m index of this wave

    for (int p0 = 0; p0 < G.n_P; p0 += FUSED_PC) {
        uint32_t Pv[FUSED_PC];
        double s11v[FUSED_PC], s12v[FUSED_PC];
#pragma unroll
        for (int p = 0; p < FUSED_PC; ++p) {
            const int pi = p0 + p < G.n_P ? p0 + p : G.n_P - 1;
            const uint32_t P = G.P[pi];
            Pv[p] = P;
            if (want_chain) {
                const int target = (int)(P - 1);
                while (j_done < target) {
                    const int block_end = (j_done / SUM_BLOCK + 1) * SUM_BLOCK;
                    const int stop = target < block_end ? target : block_end;
#pragma unroll 4
                    for (; j_done < stop; ++j_done) {
                        while (d >= w) {                       // crossed into the next interval
                            d -= w;
                            w = nxb - xb;
                            yi = nys.x;
                            sl = nys.y;
                            xb = nxb;
                            ++iv;
                            nxb = X[iv + 2];
                            nys = YS[iv + 1];
                        }
                        run = run + __builtin_fma(sl, d, yi);
                        d += md;
                    }
                    if (j_done % SUM_BLOCK == 0) {
                        done = done + run;
                        run = 0.0;
                    }
                }
            }
            s11v[p] = done + run;
            if (want_binom) {
                const int cli = ceil_log2(P);
                while (cl_done < cli) {
                    s12 = s12 + lds_gap(X, YS, n, (double)(m << cl_done));
                    ++cl_done;
                }
            }
            s12v[p] = s12;
        }

        double q[FUSED_PC], fl[FUSED_PC], clL[FUSED_PC];
        double b5[FUSED_PC];
        int i5[FUSED_PC];
#pragma unroll
        for (int p = 0; p < FUSED_PC; ++p) {
            q[p] = (double)(Pv[p] - 1);
            fl[p] = (double)floor_log2(Pv[p]);
            clL[p] = (double)ceil_log2(Pv[p]) * L;
            b5[p] = INFINITY;
            i5[p] = 0;
        }
        if (mask & (1u << 5)) {
            for (int si = 0; si < wave_nv; ++si) {             // wave-uniform
                const double sd = sS[si];
                if (sd <= limd) {                              // this lane's m admits s
                    double A, B, C;
                    segment_terms(md, sd, sR[si], sG[si], L, A, B, C);
#pragma unroll
                    for (int p = 0; p < FUSED_PC; ++p) {
                        const double T5 = __builtin_fma(q[p], C, B);
                        i5[p] = T5 < b5[p] ? si : i5[p];
                        b5[p] = min_f64(b5[p], T5);
                    }
                }
            }
        }
        // the chunk's cells go to LDS as [row][cell], then out as 64-byte runs
        if (has_b) {
            Best bc[FUSED_PC];
            int want[FUSED_PC];
            double V[FUSED_PC];
            uint32_t found[FUSED_PC];
            bool any = false;
#pragma unroll
            for (int p = 0; p < FUSED_PC; ++p) {
                const double t2 = amin < INFINITY ? __builtin_fma(q[p], amin, L) : INFINITY;
                const double t9 = amin < INFINITY ? __builtin_fma(fl[p], amin, clL[p]) : INFINITY;
                const uint32_t s5 = b5[p] < INFINITY ? (uint32_t)sS[i5[p]] : 0u;
                bc[p] = decide_bcast(mask, q[p], fl[p], (double)ceil_log2(Pv[p]), gm, L, g1, t2, 0u,
                                     b5[p], s5, t9, 0u);
                want[p] = (bc[p].id == 2u || bc[p].id == 9u) ? (int)bc[p].id : 0;
                V[p] = bc[p].t;
                found[p] = 0u;
                any = any || want[p] != 0;
            }
            if (__ballot(any) != 0) {
                first_s_of_flat_or_binomial<FUSED_PC>(
                    wave_nv, limd, md, L, q, fl, clL, want, V, found,
                    [&](int si, double &sd, double &rcp_s, double &g) {
                        sd = sS[si];
                        rcp_s = sR[si];
                        g = sG[si];
                    });
#pragma unroll
                for (int p = 0; p < FUSED_PC; ++p)
                    if (want[p] != 0)
                        bc[p].s = found[p];
            }
#pragma unroll
            for (int p = 0; p < FUSED_PC; ++p) {
                union { plogp_cell_dev c; uint4 v; } u;
                u.c.time = bc[p].t; u.c.s = bc[p].s; u.c.strategy = bc[p].id;
                stage[wave][0][lane * (FUSED_PC + 1) + p] = u.v;
            }
        }
        if (has_s) {
#pragma unroll
            for (int p = 0; p < FUSED_PC; ++p) {
                const Best r = decide_scatter(mask, q[p], (double)ceil_log2(Pv[p]), gm, L, s11v[p],
                                              s12v[p]);
                union { plogp_cell_dev c; uint4 v; } u;
                u.c.time = r.t; u.c.s = r.s; u.c.strategy = r.id;
                stage[wave][1][lane * (FUSED_PC + 1) + p] = u.v;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        {
            const int pl = lane % FUSED_PC;                    // cell within the run
            const int pi = p0 + pl;
#pragma unroll
            for (int it = 0; it < FUSED_PC; ++it) {
                const int row = it * (64 / FUSED_PC) + lane / FUSED_PC;
                const int rmi = row0 + row;
                if (rmi < G.n_m && pi < G.n_P) {
                    plogp_cell_dev *o = o_tab + (size_t)rmi * G.n_P + pi;
                    if (has_b) {
                        stream_out(o, stage[wave][0][row * (FUSED_PC + 1) + pl]);
                        o += plane;
                    }
                    if (has_s)
                        stream_out(o, stage[wave][1][row * (FUSED_PC + 1) + pl]);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// ---- whole path of one (table, m) row in one workgroup ------------------------
//
// Few candidates (one per lane of a wave) and few blocks of the Scatter-chain sum:
// a workgroup takes one (table, m) and does every step for it, with LDS between
// the steps instead of device memory and launches: the table and its slopes; wave
// 0 the candidates (g(s), k, A, B, C, min A: one lane each), wave 1 g(m), g(1)
// and the prefix of g(2^j m); all threads the terms g(j m) of the chain sum, one
// search each; wave 0 the sums inside the blocks (a lane per block, 64 dependent
// additions) and then over the blocks; then the waves run their lanes over the
// process counts as in k_sweep_p: per candidate one fma and one min for row 5 of
// Table 1, min_s A for rows 2 and 9, the winning candidate looked for only where a
// segmented row wins, two coalesced stores per cell.
constexpr int ROW_THREADS = 512;
constexpr int ROW_MAX_BLK = 32;          // at most 2048 terms of the chain sum
constexpr int ROW_NS = 64;               // candidates at most
constexpr int ROW_SPAD = ROW_NS + 8;     // the candidate loops read up to 7 entries past the last
constexpr int ROW_MAX_N = 512;           // samples at most (LDS per workgroup stays small)

static size_t row_lds_bytes(int n, int n_blk, int n_P)
{
    return ((size_t)3 * n + 3 * ROW_SPAD + 36 + 36 + (size_t)n_blk * (SUM_BLOCK + 1) + 2 * ROW_MAX_BLK +
            ROW_SPAD / 2 + (size_t)(n_P + 1) / 2) * sizeof(double);
}

// PPL: process counts per lane in the Broadcast plane.
template <bool ALL, int PPL>
__global__ void __launch_bounds__(ROW_THREADS) k_row(DeviceTables T, DeviceGrid G, plogp_cell_dev *out)
{
    extern __shared__ double lds[];
    __shared__ double sh_gm, sh_g1, sh_amin;
    __shared__ int sh_nv;
    __shared__ unsigned next_group;
    const int n = T.n, n_s = G.n_s, n_P = G.n_P, n_blk = G.n_blk;
    const uint32_t mask = ALL ? 0x1FFFu : G.mask;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // the rows of large sizes (the most candidates) first when the sizes ascend
    const int t = (int)blockIdx.x / G.n_m, mi = G.n_m - 1 - (int)blockIdx.x % G.n_m;
    double *x = lds, *y = x + n, *sl = y + n;
    double *sA = sl + n, *sB = sA + ROW_SPAD, *sC = sB + ROW_SPAD;     // per candidate
    double *sum2 = sC + ROW_SPAD, *g2 = sum2 + 36;                     // prefix of g(2^j m); its terms
    double *pre = g2 + 36;                     // [block][65]: the terms, then the sums before each
    double *tot = pre + (size_t)n_blk * (SUM_BLOCK + 1), *done = tot + ROW_MAX_BLK;
    uint32_t *sSv = reinterpret_cast<uint32_t *>(done + ROW_MAX_BLK);  // the candidates
    uint32_t *sP = sSv + ROW_SPAD;                                     // the process counts
    // everything that comes from device memory is asked for at once
    const u64 m = G.m[mi];
    const double L = T.L[t];
    const u64 my_s = wave == 0 && lane < n_s ? G.s[lane] : 0ull;
    // (the division does not wait for the table: it runs while the samples are on their way)
    const double my_sd = (double)my_s, my_rcp = 1.0 / my_sd;
    {
        const double *gx = T.x + (size_t)t * n, *gy = T.y + (size_t)t * n;
        for (int i = tid; i < n; i += ROW_THREADS) {
            x[i] = gx[i];
            y[i] = gy[i];
        }
        for (int i = tid; i < n_P; i += ROW_THREADS)
            sP[i] = G.P[i];
        if (tid == 0)
            next_group = 0u;
        __syncthreads();
        for (int i = tid; i < n; i += ROW_THREADS)
            sl[i] = interval_slope(x, y, n, i);
        __syncthreads();
    }
    const LdsTable tab = {x, y, sl, n};
    const double md = (double)m;
    const bool chain = (mask & (1u << 11)) != 0, binom = (mask & (1u << 12)) != 0;

    if (wave == 0) {
        double A = INFINITY, B = INFINITY, C = 0.0;
        bool valid = false;
        if (lane < n_s) {
            const u64 lim = m < G.s_cap ? m : G.s_cap;
            const double sd = my_sd, gs = gap_at(tab, sd);
            C = gs + L;
            valid = my_s <= lim;
            if (valid) {
                double Cx;
                segment_terms(md, sd, my_rcp, gs, L, A, B, Cx);
            }
        }
        sA[lane] = A;
        sB[lane] = B;
        sC[lane] = C;
        sSv[lane] = (uint32_t)my_s;
        if (lane < ROW_SPAD - ROW_NS) {        // past the end: never taken (B = +inf, C finite)
            sA[ROW_NS + lane] = INFINITY;
            sB[ROW_NS + lane] = INFINITY;
            sC[ROW_NS + lane] = 0.0;
            sSv[ROW_NS + lane] = 0u;
        }
        const double amin = wave_min(A);
        const int nv = __builtin_popcountll(__ballot(valid));       // the candidates ascend
        if (lane == 0) {
            sh_amin = amin;
            sh_nv = nv;
        }
    } else if (wave == 1) {
        if (binom && lane < G.cl_max)
            g2[lane] = gap_at(tab, (double)(m << lane));
        if (lane == 63) {
            sh_gm = gap_at(tab, md);
            sh_g1 = gap_at(tab, 1.0);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (binom && lane == 0) {
            double acc = 0.0;
            sum2[0] = 0.0;
            for (int j = 0; j < G.cl_max; ++j) {
                acc = acc + g2[j];
                sum2[j + 1] = acc;
            }
        }
    }
    if (chain) {
        const int n_terms = SUM_BLOCK * (n_blk - 1) + G.last_terms;
        for (int r = tid; r < n_blk * SUM_BLOCK; r += ROW_THREADS) {
            double v = 0.0;
            if (r < n_terms)
                v = gap_at(tab, (double)((u64)(r + 1) * m));
            pre[r + r / SUM_BLOCK] = v;
        }
    }
    __syncthreads();
    // wave 0 adds the chain sums up while the others start on the Broadcast plane, which
    // does not need them; it joins them afterwards (the groups of 64 process counts are
    // handed out through a counter)
    if (chain && wave == 0) {
        if (lane < n_blk) {
            // sixteen terms at a time: read, add in order, write the sums before each
            double *p = pre + lane * (SUM_BLOCK + 1);
            double run = 0.0;
            for (int r0 = 0; r0 < SUM_BLOCK; r0 += 16) {
                double v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    v[u] = p[r0 + u];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    p[r0 + u] = run;
                    run = run + v[u];
                }
            }
            tot[lane] = run;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (lane == 0) {
            double acc = 0.0;
            for (int b = 0; b < n_blk; ++b) {      // the finished blocks, in ascending order
                done[b] = acc;
                acc = acc + tot[b];
            }
        }
    }

    const double gm = sh_gm, g1 = sh_g1, amin = sh_amin;
    const int nv = sh_nv;
    const size_t plane = (size_t)G.n_m * n_P;
    plogp_cell_dev *const orow = out + (size_t)t * G.n_ops * plane + (size_t)mi * n_P;
    // lane si keeps C of candidate si (lanes past the candidates: 0, never taken as B is +inf)
    const double c_mine = sC[lane];
    const int c_lo = __double2loint(c_mine), c_hi = __double2hiint(c_mine);
    // a lane takes PPL process counts, 64 apart: a candidate read from LDS serves them all
    const unsigned n_groups = (unsigned)((n_P + 64 * PPL - 1) / (64 * PPL));
    if (mask & 0x3FFu) {
        for (;;) {
            unsigned grp = 0u;
            if (lane == 0)
                grp = atomicAdd(&next_group, 1u);
            grp = __builtin_amdgcn_readfirstlane(grp);
            if (grp >= n_groups)
                break;
            int pi[PPL];
            bool active[PPL];
            double q[PPL], fl[PPL], cl[PPL], clL[PPL], b5[PPL];
            int i5[PPL];
#pragma unroll
            for (int h = 0; h < PPL; ++h) {
                pi[h] = ((int)grp * PPL + h) * 64 + lane;
                active[h] = pi[h] < n_P;
                const uint32_t Pv = sP[active[h] ? pi[h] : n_P - 1];
                q[h] = (double)(Pv - 1u);
                fl[h] = (double)floor_log2(Pv);
                cl[h] = (double)ceil_log2(Pv);
                clL[h] = cl[h] * L;
                b5[h] = INFINITY;
                i5[h] = 0;
            }
            // row 5: min over s of fma(q, C, B), eight candidates per round trip to LDS; the
            // batch in which the minimum first appeared is remembered
            if (mask & 0x20u) {
                for (int s0 = 0; s0 < nv; s0 += 8) {
                    // B from LDS (the same address in every lane), C from the lane that holds
                    // it, through scalar registers: half the LDS traffic
                    double Bv[8], Cv[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        Bv[u] = sB[s0 + u];
                        Cv[u] = __hiloint2double(__builtin_amdgcn_readlane(c_hi, s0 + u),
                                                 __builtin_amdgcn_readlane(c_lo, s0 + u));
                    }
#pragma unroll
                    for (int h = 0; h < PPL; ++h) {
                        double cur = INFINITY;
#pragma unroll
                        for (int u = 0; u < 8; ++u)
                            cur = min_f64(cur, __builtin_fma(q[h], Cv[u], Bv[u]));
                        i5[h] = cur < b5[h] ? s0 : i5[h];
                        b5[h] = min_f64(b5[h], cur);
                    }
                }
            }
#pragma unroll
            for (int h = 0; h < PPL; ++h) {
                const double t2 = amin < INFINITY ? __builtin_fma(q[h], amin, L) : INFINITY;
                const double t9 = amin < INFINITY ? __builtin_fma(fl[h], amin, clL[h]) : INFINITY;
                Best bc = decide_bcast(mask, q[h], fl[h], cl[h], gm, L, g1, t2, 0u, b5[h], 0u, t9, 0u);
                if (__ballot(active[h] && bc.id == 5u) != 0) {
                    // the first candidate of the remembered batch that attains the minimum
                    int at5 = i5[h];
#pragma unroll
                    for (int u = 7; u >= 0; --u)        // descending: the first match stays
                        at5 = __builtin_fma(q[h], sC[i5[h] + u], sB[i5[h] + u]) == b5[h] ? i5[h] + u : at5;
                    const uint32_t s_at = sSv[at5];
                    bc.s = bc.id == 5u ? s_at : bc.s;
                }
                bool open = active[h] && (bc.id == 2u || bc.id == 9u);
                if (__ballot(open) != 0) {
                    // a winning row 2 or 9: the first candidate whose value equals the minimum
                    const double mul = bc.id == 2u ? q[h] : fl[h], add = bc.id == 2u ? L : clL[h];
                    uint32_t found = 0u;
                    for (int s0 = 0; s0 < nv; s0 += 4) {     // past the last candidate A is +inf
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const bool hit = open && __builtin_fma(mul, sA[s0 + u], add) == bc.t;
                            found = hit ? sSv[s0 + u] : found;
                            open = open && !hit;
                        }
                        if (__ballot(open) == 0)
                            break;
                    }
                    if (bc.id == 2u || bc.id == 9u)
                        bc.s = found;
                }
                if (active[h])
                    store_cell(orow + pi[h], bc);
            }
        }
    }
    __syncthreads();                   // the chain sums are complete
    if (mask & 0x1C00u) {
        plogp_cell_dev *const srow = orow + ((mask & 0x3FFu) ? plane : 0);
        for (int pi = tid; pi < n_P; pi += ROW_THREADS) {
            const uint32_t Pv = sP[pi];
            const int cli = ceil_log2(Pv), blk = (int)((Pv - 1u) / SUM_BLOCK);
            const double s11 = chain ? done[blk] + pre[(Pv - 1u) + blk] : 0.0;
            const double s12 = binom ? sum2[cli] : 0.0;
            store_cell(srow + pi, decide_scatter(mask, (double)(Pv - 1u), (double)cli, gm, L, s11, s12));
        }
    }
}

// ---- whole path for batches of tables that share their sample sizes ----------
//
// Measured tables of many clusters are normally taken at the same list of
// message sizes.  Then, for a fixed m, everything that depends on where a size
// falls among the samples -- the interval of m, of 2^j m, of every j m of the
// Scatter-chain sum, the candidates that compete, k = ceil(m / s) -- is the same
// for all tables, and only the gaps, slopes and L differ.  So here the lanes of a
// wave run over 64 tables and the wave walks over message sizes: all control
// flow is wave-uniform (no lane ever waits for another lane's interval
// crossing), the table entries are read as coalesced rows of a copy laid out
// [interval][table], and the per-m facts come from small tables prepared once
// per call by k_batch_setup.

// One thread per entry of the prepared facts.  Uses table 0's sample sizes.
// Intervals are numbered as in the chain walk: 0 = [0, x_0) (the clamp: gap y_0,
// slope 0), i + 1 = [x_i, x_{i+1}), n = [x_{n-1}, inf).  Everything about one
// message size sits in one record of B.rec (layout: BatchRec).
__device__ __forceinline__ void batch_prep_body(const DeviceTables &T, const DeviceGrid &G,
                                                const BatchPrep &B, int block, int n_blocks, double *lds)
{
    const int n = T.n;
    double *x = lds;                              // samples of table 0
    for (int i = threadIdx.x; i < n; i += blockDim.x)
        x[i] = T.x[i];
    __syncthreads();
    // interval of size z and z minus the start of that interval (exact)
    auto locate = [&](double z, int &iv, double &dz) {
        const int cnt = last_not_above(x, n, z) + (z >= x[0] ? 1 : 0);     // samples not above z
        iv = cnt;
        dz = cnt == 0 ? z : z - x[cnt - 1];
    };
    const BatchRec R(n, G.n_s, G.cl_max);
    const long tid = (long)block * blockDim.x + threadIdx.x;
    const long stride = (long)n_blocks * blockDim.x;
    for (long e = tid; e < G.n_m; e += stride) {
        double *rec = B.rec + (size_t)e * R.slots;
        const u64 m = G.m[e];
        int iv;
        double dz;
        locate((double)m, iv, dz);
        const u64 lim = m < G.s_cap ? m : G.s_cap;          // candidates s <= min(m, s_cap) ascend
        int lo = 0, hi = G.n_s;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (G.s[mid] <= lim) lo = mid + 1; else hi = mid;
        }
        rec[R.DM] = dz;
        rec[R.MD] = (double)m;
        reinterpret_cast<int *>(rec + R.IM_NV)[0] = iv;
        reinterpret_cast<int *>(rec + R.IM_NV)[1] = lo;
    }
    for (long e = tid; e < (long)G.n_m * G.cl_max; e += stride) {
        const long mi = e / G.cl_max;
        const int j = (int)(e % G.cl_max);
        double *rec = B.rec + (size_t)mi * R.slots;
        int iv;
        double dz;
        locate((double)(G.m[mi] << j), iv, dz);
        rec[R.D2 + j] = dz;
        reinterpret_cast<int *>(rec + R.I2)[j] = iv;
    }
    for (long e = tid; e < (long)G.n_m * (n + 1); e += stride) {
        // last j whose size j m still lies in interval i of this m: below the next sample
        const long mi = e / (n + 1);
        const int i = (int)(e % (n + 1));
        const u64 m = G.m[mi];
        u64 last = 0xFFFFFFFFull;
        if (i < n) {
            last = ((u64)x[i] - 1ull) / m;
            last = last < 0xFFFFFFFFull ? last : 0xFFFFFFFFull;
        }
        reinterpret_cast<unsigned *>(B.rec + (size_t)mi * R.slots + R.JEND)[i] = (unsigned)last;
    }
    for (long e = tid; e < (long)G.n_m * G.n_s; e += stride) {
        const long mi = e / G.n_s;
        const int si = (int)(e % G.n_s);
        const u64 m = G.m[mi], sv = G.s[si];
        B.rec[(size_t)mi * R.slots + R.K + si] = (double)((m + sv - 1ull) / sv);   // k = ceil(m / s), exact
    }
    // B.tab: interval of size 1 and 1 minus its start; widths of the intervals; per candidate
    // s minus the start of its interval, then its interval; per process count three doubles
    for (long e = tid; e < G.n_s; e += stride) {
        int iv;
        double dz;
        locate((double)G.s[e], iv, dz);
        B.tab[2 + (n + 1) + e] = dz;
        B.tab[2 + (n + 1) + G.n_s + e] = (double)iv;
    }
    for (long e = tid; e <= n; e += stride)
        B.tab[2 + e] = e == 0 ? x[0] : (e < n ? x[e] - x[e - 1] : INFINITY);
    // per process count 32 bytes: P - 1, floor(log2 P), ceil(log2 P) as doubles, then P - 1 and
    // ceil(log2 P) as integers; the list is filled up to a multiple of eight, plus one, with
    // copies of its last entry (the kernel takes eight at a time and fetches one ahead)
    for (long e = tid; e < batch_padded_P(G.n_P); e += stride) {
        double *pt = B.tab + 2 + (n + 1) + 2 * (size_t)G.n_s + 4 * e;
        const uint32_t P = G.P[e < G.n_P ? e : G.n_P - 1];
        pt[0] = (double)(P - 1u);
        pt[1] = (double)floor_log2(P);
        pt[2] = (double)ceil_log2(P);
        reinterpret_cast<uint32_t *>(pt + 3)[0] = P - 1u;
        reinterpret_cast<uint32_t *>(pt + 3)[1] = (uint32_t)ceil_log2(P);
    }
    if (tid == 0) {
        int i1;
        double d1;
        locate(1.0, i1, d1);
        B.tab[0] = (double)i1;
        B.tab[1] = d1;
    }
}

// The tables laid out by interval: ysT[i][t] = {gap, slope} of interval i of table t
// (i = 0: the clamp {y_0, 0}; i = n + 1: zeros, only ever fetched ahead).  The slopes
// are formed here from the raw samples.  A workgroup takes BATCH_STAGE_TT tables: their
// gaps are read as whole rows into LDS (rows padded by one), then written with the
// tables along the lanes.  The sample sizes are those of table 0 (shared by all).
constexpr int BATCH_STAGE_TT = 32;

__device__ __forceinline__ void batch_stage_body(const DeviceTables &T, f64x2 *ysT, int block, double *lds)
{
    const int n = T.n, t0 = block * BATCH_STAGE_TT;
    const int nt = T.n_tables - t0 < BATCH_STAGE_TT ? T.n_tables - t0 : BATCH_STAGE_TT;
    for (int e = threadIdx.x; e < nt * n; e += blockDim.x) {
        const int tl = e / n, i = e - tl * n;
        lds[tl * (n + 1) + i] = T.y[(size_t)(t0 + tl) * n + i];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < (n + 2) * BATCH_STAGE_TT; e += blockDim.x) {
        const int i = e / BATCH_STAGE_TT, tl = e % BATCH_STAGE_TT;
        if (tl >= nt)
            continue;
        const double *y = lds + tl * (n + 1);
        f64x2 v = {0.0, 0.0};
        if (i == 0)
            v = f64x2{y[0], 0.0};
        else if (i <= n)
            v = f64x2{y[i - 1], interval_slope(T.x, y, n, i - 1)};
        ysT[(size_t)i * T.n_tables + t0 + tl] = v;
    }
}

// One launch for both preparations: the first n_stage workgroups lay out the tables, the
// others prepare the per-size facts.
__global__ void __launch_bounds__(256) k_batch_setup(DeviceTables T, DeviceGrid G, BatchPrep B,
                                                     f64x2 *ysT, int n_stage)
{
    extern __shared__ double lds[];
    if ((int)blockIdx.x < n_stage)
        batch_stage_body(T, ysT, (int)blockIdx.x, lds);
    else
        batch_prep_body(T, G, B, (int)blockIdx.x - n_stage, (int)gridDim.x - n_stage, lds);
}

constexpr size_t BATCH_T_LDS_MAX = 160 * 1024;     // LDS of a compute unit

// A wave-uniform read of data that no kernel writes while this one runs, through the
// scalar cache (constant address space).  Unlike a vector load it does not queue behind
// the wave's outstanding stores.
template <class V>
__device__ __forceinline__ V uniform_load(const V *p)
{
    typedef const V __attribute__((address_space(4))) *const_ptr;
    return *(const_ptr)(p);
}
constexpr int BATCH_T_WAVES = 16;      // waves of a workgroup; they share the 64 tables
constexpr int BATCH_T_PC = 4;          // process counts decided together (in registers)
constexpr int BATCH_T_PS = 8;          // process counts per pass over the candidates, and the
                                       // cells of a table written together (128 bytes)
// Output staging of a wave, used in turn as 64 rows of 8 times + 8 one-byte ids (Scatter)
// and as 32 rows of 8 cells padded to 9 (Broadcast).
constexpr int BATCH_T_STAGE = 64 * 72;
static_assert(BATCH_T_STAGE >= 32 * (BATCH_T_PS + 1) * 16 && BATCH_T_STAGE % 16 == 0, "both layouts fit");

struct BatchDims {
    int n, n_tables, n_m, n_P, n_s, cl_max, n_ops, n_mchunks, m_per_wave;
    uint32_t mask;
    uint32_t extra;   // rows beyond the tables: bits 0..2 Gather, bits 3, 4 Barrier (see DeviceGrid)
};

// A workgroup stages its 64 tables by interval in LDS (YS[i][lane] = {gap, slope}
// of interval i of the lane's table) together with their g(s); every later
// access to a table is one conflict-free LDS read of a whole row.  All other
// inputs are wave-uniform and come through the scalar cache.  The cells of PS = 8
// process counts are turned round in LDS so that eight neighbouring lanes store
// the 128 contiguous bytes of one table (whole cache lines when n_P is a multiple
// of 8: measured 5.2 TB/s against 3.3 TB/s for 64-byte runs).  LDS has room for
// 4.5 KB of staging per wave, not for 64 rows of 8 cells: a Scatter cell is staged
// as its time and a one-byte id (s is 0), the Broadcast cells go out in two halves
// of 32 tables, the second half waiting in registers.
// ALL: every strategy of Tables 1 and 2 is enabled (the mask is a compile-time constant).
// EXTRA: rows beyond the tables are enabled as well (their planes cost nothing otherwise).
template <int PC, int PS, bool ALL, bool EXTRA>
__global__ void __launch_bounds__(64 * BATCH_T_WAVES)
k_batch_t(BatchDims D, const f64x2 *__restrict__ ysT, const double *__restrict__ Lt,
          const double *__restrict__ recs, const double *__restrict__ tab,
          const u64 *__restrict__ p_s, plogp_cell_dev *__restrict__ out)
{
    extern __shared__ __align__(16) double batch_lds[];
    const int n = D.n, n_s = D.n_s, n_P = D.n_P;
    const BatchRec R(n, n_s, D.cl_max);
    f64x2 *YS = reinterpret_cast<f64x2 *>(batch_lds);          // [n + 2][64]
    double *GS = batch_lds + (size_t)2 * (n + 2) * 64;         // [n_s][64]
    // per wave: the PC cells of 64 tables on their way out, rows padded by one cell
    char *stage_all = reinterpret_cast<char *>(GS + (size_t)(n_s ? n_s : 1) * 64);
    uint32_t *sS = reinterpret_cast<uint32_t *>(stage_all + (size_t)BATCH_T_WAVES * BATCH_T_STAGE);   // [n_s]
    unsigned &next_m = *reinterpret_cast<unsigned *>(sS + (n_s ? n_s : 1));   // next size of this workgroup's chunk
    // the chunks of large sizes (more candidates, the longest) are handed out first, so that
    // the launch ends with short workgroups
    const int n_tg = (D.n_tables + 63) / 64;
    const int tg = blockIdx.x % n_tg, mc = D.n_mchunks - 1 - (int)(blockIdx.x / n_tg);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int t = tg * 64 + lane;
    const int tc = t < D.n_tables ? t : D.n_tables - 1;
    const double L = Lt[tc];
    const uint32_t mask = ALL ? 0x1FFFu : D.mask;
    for (int si = threadIdx.x; si < n_s; si += blockDim.x)
        sS[si] = (uint32_t)p_s[si];
    for (int i = wave; i < n + 2; i += BATCH_T_WAVES)
        YS[i * 64 + lane] = ysT[(size_t)i * D.n_tables + tc];
    if (threadIdx.x == 0)
        next_m = 0u;
    __syncthreads();
    const f64x2 *ys = YS + lane;                               // this lane's table: ys[64 i]
    const double *tab_ds = tab + 2 + (n + 1), *tab_is = tab_ds + n_s, *Wd = tab + 2;
    // per process count {P - 1, floor log2 P, ceil log2 P, {P - 1, ceil log2 P} as integers}
    typedef double f64x4 __attribute__((ext_vector_type(4)));
    const f64x4 *tab_P = reinterpret_cast<const f64x4 *>(tab_is + n_s);
    for (int si = wave; si < n_s; si += BATCH_T_WAVES) {
        const f64x2 v = ys[64 * (int)uniform_load(tab_is + si)];
        GS[si * 64 + lane] = __builtin_fma(v.y, uniform_load(tab_ds + si), v.x);
    }
    double g1;
    {
        const f64x2 v = ys[64 * (int)uniform_load(tab)];
        g1 = __builtin_fma(v.y, uniform_load(tab + 1), v.x);
    }
    __syncthreads();
    const double *gsl = GS + lane;                             // g(s) of this lane's table: gsl[64 si]
    char *stage = stage_all + (size_t)wave * BATCH_T_STAGE;
    // A store instruction writes the PS cells (PS x 16 contiguous bytes) of 64 / PS tables:
    // lane l takes cell l % PS of table row l / PS + (64 / PS) it.
    static_assert(PC == 4 && PS == 8, "128-byte runs, decided four at a time");
    const int out_p = lane % PS, out_row = lane / PS;
    const size_t plane = (size_t)D.n_m * n_P;
    const size_t table_cells = (size_t)D.n_ops * plane;
    // Where the staged cells go: a wave-uniform 64-bit part (table group, row step, plane, m,
    // first process count) plus a per-lane 32-bit byte offset, so that the stores need no
    // per-lane 64-bit addresses (the host checks that the offset fits).
    const unsigned lane_off = (unsigned)(((size_t)out_row * table_cells + out_p) * sizeof(plogp_cell_dev));
    char *const o_grp = reinterpret_cast<char *>(out + (size_t)tg * 64 * table_cells);
    const int rows_left = D.n_tables - tg * 64 - out_row;      // table rows r0 + out_row with r0 < rows_left exist
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    // wave-uniform base in scalar registers + 32-bit lane offset
    auto store_run = [&](char *ubase, u32x4 cell) {
        asm volatile("global_store_dwordx4 %0, %1, %2 nt" : : "v"(lane_off), "v"(cell), "s"(ubase) : "memory");
    };
    const size_t run_step = (size_t)(64 / PS) * table_cells * sizeof(plogp_cell_dev);   // 8 tables on
    const bool whole_group = tg * 64 + 64 <= D.n_tables;       // wave-uniform: no row of tables is missing
    // cell0: index of cell (plane, mi, p0) inside a table.  Scatter layout: row r of the stage
    // holds 8 times, then 8 ids as signed bytes (-1 = no strategy).
    // id_add: 0, or 3 when the staged Scatter decisions go out as their Gather twins
    auto scatter_cell = [&](int r0, int id_add) {
        const char *row = stage + (r0 + out_row) * 72;
        const double tv = *reinterpret_cast<const double *>(row + 8 * out_p);
        const int id = *reinterpret_cast<const signed char *>(row + 64 + out_p);
        u32x4 cell;
        cell.x = (unsigned)__double2loint(tv);
        cell.y = (unsigned)__double2hiint(tv);
        cell.z = 0u;
        cell.w = (unsigned)(id < 0 ? id : id + id_add);
        return cell;
    };
    auto flush_times = [&](size_t cell0, int p0, int id_add) {
        __builtin_amdgcn_wave_barrier();
        if (p0 + out_p < n_P) {
            char *ubase = o_grp + cell0 * sizeof(plogp_cell_dev);
            if (whole_group) {
                // (four rows are read before their four stores go out: a store keeps the reads
                // that follow it behind itself)
#pragma unroll
                for (int it = 0; it < 64 / PS; it += 4) {
                    u32x4 c[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        c[u] = scatter_cell((64 / PS) * (it + u), id_add);
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        store_run(ubase, c[u]);
                        ubase += run_step;
                    }
                }
            } else {
                // (the limit is made opaque here: its sixteen compares would otherwise be kept
                // in scalar registers across the whole kernel)
                int rl = rows_left;
                asm volatile("" : "+v"(rl));
#pragma unroll
                for (int it = 0; it < 64 / PS; ++it) {
                    if ((64 / PS) * it < rl)
                        store_run(ubase, scatter_cell((64 / PS) * it, id_add));
                    ubase += run_step;
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    };
    // Broadcast layout: row r of the stage holds the 8 cells of table 32 half + r, padded to 9.
    auto flush_cells = [&](int half, size_t cell0, int p0) {
        __builtin_amdgcn_wave_barrier();
        if (p0 + out_p < n_P) {
            char *ubase = o_grp + ((size_t)32 * half * table_cells + cell0) * sizeof(plogp_cell_dev);
            const u32x4 *rows = reinterpret_cast<const u32x4 *>(stage) + out_row * (PS + 1) + out_p;
            if (whole_group) {
                u32x4 c[32 / PS];
#pragma unroll
                for (int it = 0; it < 32 / PS; ++it)
                    c[it] = rows[(64 / PS) * it * (PS + 1)];
#pragma unroll
                for (int it = 0; it < 32 / PS; ++it) {
                    store_run(ubase, c[it]);
                    ubase += run_step;
                }
            } else {
                int rl = rows_left;
                asm volatile("" : "+v"(rl));
#pragma unroll
                for (int it = 0; it < 32 / PS; ++it) {
                    if (32 * half + (64 / PS) * it < rl)
                        store_run(ubase, rows[(64 / PS) * it * (PS + 1)]);
                    ubase += run_step;
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    };
    auto pack = [](const Best &b) {
        union { plogp_cell_dev c; uint4 v; } u;
        u.c.time = b.t; u.c.s = b.s; u.c.strategy = b.id;
        return u.v;
    };
    // The Gather rows (ids 13..15) are the Scatter rows on the same sums: this kernel takes them
    // when they are enabled exactly as the Scatter rows are, or without any Scatter row (the host
    // sees to that), decides once and writes the decisions to both planes.  The Barrier rows
    // (16, 17) need g(1), L and the process count only.
    const uint32_t extra = EXTRA ? D.extra : 0u;
    const uint32_t gather_rows = (extra & 7u) << 10;               // as the Scatter rows they mirror
    const uint32_t sg_rows = (mask & 0x1C00u) | gather_rows;
    const bool want_chain = (sg_rows & (1u << 11)) != 0, want_binom = (sg_rows & (1u << 12)) != 0;
    const bool has_b = (mask & 0x3FFu) != 0, has_s = sg_rows != 0;
    const bool has_scatter = (mask & 0x1C00u) != 0, has_gather = gather_rows != 0;
    const bool has_barrier = (extra & 0x18u) != 0;
    const size_t scatter_at = (has_b ? plane : 0), gather_at = scatter_at + (has_scatter ? plane : 0);
    const size_t barrier_at = gather_at + (has_gather ? plane : 0);

    // The waves take the sizes of the workgroup's chunk one at a time from a counter, the largest
    // first (a size's cost grows with its number of candidates): the one workgroup that fits a
    // compute unit then ends with all its waves busy, whatever the mix.
    const int chunk = BATCH_T_WAVES * D.m_per_wave;
    for (;;) {
        unsigned k = 0u;
        if (lane == 0)
            k = atomicAdd(&next_m, 1u);
        k = (unsigned)__builtin_amdgcn_readfirstlane((int)k);
        if (k >= (unsigned)chunk)
            break;
        const int mi = mc * chunk + chunk - 1 - (int)k;                      // wave-uniform
        if (mi >= D.n_m)
            continue;
        const double *rec = recs + (size_t)mi * R.slots;
        const double md = uniform_load(rec + R.MD);
        const int nvm = uniform_load(reinterpret_cast<const int *>(rec + R.IM_NV) + 1);
        const double *Krow = rec + R.K;
        const unsigned *jend = reinterpret_cast<const unsigned *>(rec + R.JEND);
        // g(m); the chain sum starts at j = 1 in the same interval
        int ci = uniform_load(reinterpret_cast<const int *>(rec + R.IM_NV));
        f64x2 cur = ys[64 * ci];
        double d = uniform_load(rec + R.DM);                    // size - start of its interval
        const double gm = __builtin_fma(cur.y, d, cur.x);
        unsigned je = uniform_load(jend + ci);                  // last j inside interval ci
        // fetched one crossing ahead: the next interval's entries, its last j, this one's width
        f64x2 nxt = ys[64 * (ci + 1)];
        unsigned je_n = uniform_load(jend + (ci < n ? ci + 1 : n));
        double w_n = uniform_load(Wd + ci);
        double run = 0.0, done = 0.0;
        unsigned j_done = 0;
        double s12 = 0.0;
        int cl_done = 0;
        int i2_n = uniform_load(reinterpret_cast<const int *>(rec + R.I2));
        double d2_n = uniform_load(rec + R.D2);
        f64x4 P_n = uniform_load(tab_P);
        // minimum over s of A = g(s) k (rows 2 and 9 of Table 1 are monotone in A), the first
        // candidate that attains it, and the least A before that candidate (+inf if none)
        double amin = INFINITY, abefore = INFINITY;
        int imin = 0;
        if (mask & 0x204u) {
            // (the next candidate's g(s) and k are fetched while this one is worked on)
            double gs_n = gsl[0], k_n = uniform_load(Krow);
            for (int si = 0; si < nvm; ++si) {
                const double A = gs_n * k_n;
                const int nx = si + 1 < nvm ? si + 1 : si;
                gs_n = gsl[64 * nx];
                k_n = uniform_load(Krow + nx);
                const bool lower = A < amin;
                abefore = lower ? amin : abefore;
                imin = lower ? si : imin;
                amin = min_f64(amin, A);
            }
        }

        // PS process counts per pass over the candidates (the per-candidate terms are formed
        // once for all of them), then PC cells at a time are decided and written
        for (int q0 = 0; q0 < n_P; q0 += PS) {
            const size_t cell0 = (size_t)mi * n_P + q0;
            if (has_s) {
                // Scatter plane, one process count after the other: the chain sum is walked
                // along j while P ascends, the binomial sum grows with ceil(log2 P)
#pragma nounroll
                for (int p = 0; p < PS; ++p) {
                    const f64x4 Pv = P_n;                       // (fetched one step ahead, like i2_n and d2_n)
                    P_n = uniform_load(tab_P + q0 + p + 1);
                    if (want_chain) {
                        const unsigned target = (unsigned)__double2loint(Pv.w);
                        while (j_done < target) {
                            // up to the next process count, block end or interval end
                            const unsigned block_end = (j_done / SUM_BLOCK + 1u) * SUM_BLOCK;
                            unsigned stop = target < block_end ? target : block_end;
                            stop = stop < je ? stop : je;
                            unsigned j = j_done;
                            for (; j + 4u <= stop; j += 4u) {
#pragma unroll
                                for (int r = 0; r < 4; ++r) {
                                    run = run + __builtin_fma(cur.y, d, cur.x);
                                    d += md;
                                }
                            }
                            for (; j < stop; ++j) {
                                run = run + __builtin_fma(cur.y, d, cur.x);
                                d += md;
                            }
                            j_done = stop;
                            if (j_done % SUM_BLOCK == 0u) {
                                done = done + run;
                                run = 0.0;
                            }
                            while (je <= j_done) {              // the next size lies further on
                                d -= w_n;
                                ++ci;
                                cur = nxt;
                                je = je_n;
                                nxt = ys[64 * (ci + 1)];
                                je_n = uniform_load(jend + (ci < n ? ci + 1 : n));
                                w_n = uniform_load(Wd + ci);
                            }
                        }
                    }
                    if (want_binom) {
                        const int cli = __double2hiint(Pv.w);
                        while (cl_done < cli) {
                            const f64x2 v = ys[64 * i2_n];
                            s12 = s12 + __builtin_fma(v.y, d2_n, v.x);
                            ++cl_done;
                            const int nx = cl_done < D.cl_max ? cl_done : cl_done - 1;
                            i2_n = uniform_load(reinterpret_cast<const int *>(rec + R.I2) + nx);
                            d2_n = uniform_load(rec + R.D2 + nx);
                        }
                    }
                    const Best r = decide_scatter(ALL ? mask : sg_rows, Pv.x, Pv.z, gm, L, done + run, s12);
                    *reinterpret_cast<double *>(stage + lane * 72 + 8 * p) = r.t;
                    *reinterpret_cast<signed char *>(stage + lane * 72 + 64 + p) = (signed char)r.id;
                }
                if (has_scatter)
                    flush_times(scatter_at + cell0, q0, 0);
                if (has_gather)
                    flush_times(gather_at + cell0, q0, 3);
            }
            if (has_barrier) {
                // twice the flat-tree and the binomial row of Table 1 at one byte; the same for
                // every message size, formed again for each (what it would take to keep them
                // costs more than the few instructions)
#pragma unroll
                for (int p = 0; p < PS; ++p) {
                    const f64x4 Pv = uniform_load(tab_P + q0 + p);
                    Best b = {INFINITY, 0u, 0xFFFFFFFFu};
                    if (extra & 8u) consider(b, 2.0 * __builtin_fma(Pv.x, g1, L), 16, 0);
                    if (extra & 16u) consider(b, 2.0 * __builtin_fma(Pv.y, g1, Pv.z * L), 17, 0);
                    *reinterpret_cast<double *>(stage + lane * 72 + 8 * p) = b.t;
                    *reinterpret_cast<signed char *>(stage + lane * 72 + 64 + p) = (signed char)b.id;
                }
                flush_times(barrier_at + cell0, q0, 0);
            }
            if (!has_b)
                continue;
            double b5[PS];
            int i5[PS];
#pragma unroll
            for (int p = 0; p < PS; ++p) {
                b5[p] = INFINITY;
                i5[p] = 0;
            }
            if (has_b && (mask & (1u << 5))) {
                double q[PS];                                   // wave-uniform
#pragma unroll
                for (int p = 0; p < PS; ++p)
                    q[p] = uniform_load(reinterpret_cast<const double *>(tab_P + q0 + p));
                double gs_n = gsl[0], k_n = uniform_load(Krow);
                for (int si = 0; si < nvm; ++si) {
                    const double gs = gs_n, k = k_n;
                    const int nx = si + 1 < nvm ? si + 1 : si;
                    gs_n = gsl[64 * nx];
                    k_n = uniform_load(Krow + nx);
                    const double Bv = gs * (k - 1.0), Cv = gs + L;
#pragma unroll
                    for (int p = 0; p < PS; ++p) {
                        const double T5 = __builtin_fma(q[p], Cv, Bv);
                        i5[p] = T5 < b5[p] ? si : i5[p];
                        b5[p] = min_f64(b5[p], T5);
                    }
                }
            }
            Best held[PC];                                      // the first four cells of tables 32..63
#pragma unroll
            for (int g = 0; g < PS / PC; ++g) {
                const int p0 = q0 + g * PC;                     // may lie past the end: indices are clamped
                double q[PC], fl[PC], clL[PC], cl[PC];          // q, fl, cl: wave-uniform
#pragma unroll
                for (int p = 0; p < PC; ++p) {
                    const double *pt = reinterpret_cast<const double *>(tab_P + p0 + p);
                    q[p] = uniform_load(pt);
                    fl[p] = uniform_load(pt + 1);
                    cl[p] = uniform_load(pt + 2);
                    clL[p] = cl[p] * L;
                }
                Best bc[PC];
                bool any = false;
#pragma unroll
                for (int p = 0; p < PC; ++p) {
                    // without a candidate amin is +inf, and so are both values (q, fl >= 1)
                    const double t2 = __builtin_fma(q[p], amin, L);
                    const double t9 = __builtin_fma(fl[p], amin, clL[p]);
                    const double t5 = b5[g * PC + p];
                    const uint32_t s5 = t5 < INFINITY ? sS[i5[g * PC + p]] : 0u;
                    bc[p] = decide_bcast(mask, q[p], fl[p], cl[p], gm, L, g1, t2, 0u, t5, s5, t9, 0u);
                    any = any || bc[p].id == 2u || bc[p].id == 9u;
                }
                if (__ballot(any) != 0) {
                    // A winning row 2 or 9: the first candidate whose value equals the minimum.
                    // The rows grow with A, so that is the candidate of the least A, unless a
                    // larger A before it rounds to the same time: only the least of those can.
                    bool open[PC];
                    bool tie = false;
                    const uint32_t smin = nvm > 0 ? sS[imin] : 0u;
#pragma unroll
                    for (int p = 0; p < PC; ++p) {
                        open[p] = bc[p].id == 2u || bc[p].id == 9u;
                        const double Tb = bc[p].id == 2u ? __builtin_fma(q[p], abefore, L)
                                                         : __builtin_fma(fl[p], abefore, clL[p]);
                        tie = tie || (open[p] && Tb == bc[p].t);
                        bc[p].s = open[p] ? smin : bc[p].s;
                    }
                    if (__ballot(tie) != 0) {
                        // (rare) the search itself, for every lane
                        for (int si = 0; si < nvm; ++si) {
                            const double A = gsl[64 * si] * uniform_load(Krow + si);
                            const uint32_t sv = sS[si];
#pragma unroll
                            for (int p = 0; p < PC; ++p) {
                                const double Tv = bc[p].id == 2u ? __builtin_fma(q[p], A, L)
                                                                 : __builtin_fma(fl[p], A, clL[p]);
                                if (open[p] && Tv == bc[p].t) {
                                    bc[p].s = sv;
                                    open[p] = false;
                                }
                            }
                        }
                    }
                }
                uint4 *rows = reinterpret_cast<uint4 *>(stage);
                if (g == 0) {
                    if (lane < 32) {
#pragma unroll
                        for (int p = 0; p < PC; ++p)
                            rows[lane * (PS + 1) + p] = pack(bc[p]);
                    }
#pragma unroll
                    for (int p = 0; p < PC; ++p)
                        held[p] = bc[p];
                } else {
                    if (lane < 32) {
#pragma unroll
                        for (int p = 0; p < PC; ++p)
                            rows[lane * (PS + 1) + PC + p] = pack(bc[p]);
                    }
                    flush_cells(0, cell0, q0);
                    if (lane >= 32) {
#pragma unroll
                        for (int p = 0; p < PC; ++p) {
                            rows[(lane - 32) * (PS + 1) + p] = pack(held[p]);
                            rows[(lane - 32) * (PS + 1) + PC + p] = pack(bc[p]);
                        }
                    }
                    flush_cells(1, cell0, q0);
                }
            }
        }
    }
}

// ---- prediction against measurement ------------------------------------------
//
// The step after the tuning in the paper (Section 4): every implementation is
// measured, the measurements are set against the predictions of Tables 1 and
// 2, and the question is whether the technique the models choose is the one
// that is fastest in the measurement.  k_score: one thread per (m, P), lanes
// along P (the measured times meas[r][m][P] and the predictions are read and
// written coalesced); r runs over the enabled strategies in ascending id.
// g(m), g(1) and the two Scatter sums come from the tuning's own first stages.

struct plogp_verdict_dev {
    double regret;
    uint32_t pred_best;
    uint32_t meas_best;
};

// The prediction of strategy `id` (rows of Tables 1 and 2 as the scoring evaluates them) at one
// point: a segmented row at the segment size the point was measured with (gs, k; NaN if that
// size is not usable), the Scatter rows from the tuning's sums.
__device__ __forceinline__ double score_predict(int id, double q, double fl, double cl, double gm, double L,
                                                double R, const double (&gs)[3], const double (&k)[3],
                                                const bool (&ok)[3], const DeviceGrid &G, const Scratch &S,
                                                int mi, int pi, uint32_t P)
{
    switch (id) {
    case 0: case 10: return __builtin_fma(q, gm, L);
    case 1: return __builtin_fma(q, gm, R);
    case 2: return ok[0] ? __builtin_fma(q, gs[0] * k[0], L) : NAN;
    case 3: return q * (gm + L);
    case 4: return q * (gm + R);
    case 5: return ok[1] ? __builtin_fma(q, gs[1] + L, gs[1] * (k[1] - 1.0)) : NAN;
    case 6: return cl * __builtin_fma(2.0, gm, L);
    case 7: return __builtin_fma(fl, gm, cl * L);
    case 8: return __builtin_fma(fl, gm, cl * R);
    case 9: return ok[2] ? __builtin_fma(fl, gs[2] * k[2], cl * L) : NAN;
    case 11: return __builtin_fma(q, L, chain_sum_of(G, S, 0, mi, pi, P));
    default: return __builtin_fma(cl, L, S.sum2[(size_t)mi * (G.cl_max + 1) + ceil_log2(P)]);
    }
}

// Workgroups walk the (m, chunk of P) items with a stride, so that a big table is
// staged once per workgroup; the measured times and segment sizes of a point are
// fetched before any arithmetic (13 + 3 independent loads per lane in flight).
__global__ void __launch_bounds__(1024) k_score_points(DeviceTables T, DeviceGrid G, Scratch S,
                                                const double *__restrict__ meas,
                                                const uint32_t *__restrict__ seg,
                                                double *__restrict__ pred,
                                                plogp_verdict_dev *__restrict__ verdict, int n_pchunks,
                                                int n_items)
{
    extern __shared__ double lds[];
    const uint32_t mask = G.mask;
    const bool any_seg = (mask & 0x224u) != 0;
    LdsTable tab = {nullptr, nullptr, nullptr, T.n};
    if (any_seg)
        tab = stage_table(lds, T, 0);                 // for g(s) at the measured segment sizes
    const double L = T.L[0];
    const double g1 = S.g1[0];
    const double R = __builtin_fma(3.0, L, 2.0 * g1);
    const size_t plane = (size_t)G.n_m * G.n_P;
    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int mi = item / n_pchunks;
        const int pi = (item % n_pchunks) * blockDim.x + threadIdx.x;
        if (pi >= G.n_P)
            continue;
        const size_t cell = (size_t)mi * G.n_P + pi;
        double tm[13];
        uint32_t sv[3] = {0u, 0u, 0u};
        {
            int r = 0;
#pragma unroll
            for (int id = 0; id < 13; ++id) {
                tm[id] = 0.0;
                if ((mask >> id) & 1u) {
                    const size_t at = (size_t)r * plane + cell;
                    tm[id] = meas[at];
                    if (id == 2) sv[0] = seg[at];
                    if (id == 5) sv[1] = seg[at];
                    if (id == 9) sv[2] = seg[at];
                    ++r;
                }
            }
        }
        const u64 m = G.m[mi];
        const uint32_t P = G.P[pi];
        const double q = (double)(P - 1), fl = (double)floor_log2(P), cl = (double)ceil_log2(P);
        const double gm = S.gm[mi];
        double gs[3] = {0.0, 0.0, 0.0}, k[3] = {0.0, 0.0, 0.0};
        bool ok[3] = {true, true, true};
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            if (!((mask >> (u == 0 ? 2 : u == 1 ? 5 : 9)) & 1u))
                continue;
            const u64 sz = sv[u];
            ok[u] = sz > 0 && sz <= m;
            if (ok[u]) {
                gs[u] = gap_at(tab, (double)sz);
                k[u] = segments(m, sz);
            }
        }
        double best_p[2] = {INFINITY, INFINITY}, best_m[2] = {INFINITY, INFINITY};
        double meas_of_pred_best[2] = {NAN, NAN};
        uint32_t id_p[2] = {0xFFFFFFFFu, 0xFFFFFFFFu}, id_m[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};
        int r = 0;
#pragma unroll
        for (int id = 0; id < 13; ++id) {
            if (!((mask >> id) & 1u))
                continue;
            const size_t at = (size_t)r * plane + cell;
            ++r;
            const double v = score_predict(id, q, fl, cl, gm, L, R, gs, k, ok, G, S, mi, pi, P);
            __builtin_nontemporal_store(v, pred + at);
            const double t_meas = tm[id];
            const int op = id < 10 ? 0 : 1;
            if (v < best_p[op]) {
                best_p[op] = v;
                id_p[op] = (uint32_t)id;
                meas_of_pred_best[op] = t_meas;
            }
            if (t_meas < best_m[op]) {
                best_m[op] = t_meas;
                id_m[op] = (uint32_t)id;
            }
        }
        plogp_verdict_dev *o = verdict + cell;
#pragma unroll
        for (int op = 0; op < 2; ++op) {
            if (!(mask & (op == 0 ? 0x3FFu : 0x1C00u)))
                continue;
            union {
                plogp_verdict_dev vd;
                uint4 v;
            } u;
            u.vd.regret = meas_of_pred_best[op] / best_m[op] - 1.0;
            u.vd.pred_best = id_p[op];
            u.vd.meas_best = id_m[op];
            stream_out(o, u.v);
            o += plane;
        }
    }
}

// e = |(pred - meas) / meas| per point; per (strategy row r, m): the sum over P in
// ascending order from +0.0 and the maximum.  rows[(r * n_m + mi) * 2] = {sum, max}.
// A wave takes SCORE_RT rows of n_P points: per chunk of 64 process counts every lane
// loads one point of each row (coalesced) and leaves e in LDS; then lane i < SCORE_RT
// adds the 64 values of row i in order, while the loads of the next chunk are in
// flight.  The running sums stay in those lanes.
constexpr int SCORE_RT = 8;
constexpr int SCORE_WAVES = 4;

__global__ void __launch_bounds__(64 * SCORE_WAVES) k_score_rows(DeviceGrid G, int n_ids,
                                                                  const double *__restrict__ meas,
                                                                  const double *__restrict__ pred,
                                                                  double *__restrict__ rows)
{
    __shared__ double tile[SCORE_WAVES][SCORE_RT][65];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const long n_rows = (long)n_ids * G.n_m;
    const long row0 = ((long)blockIdx.x * SCORE_WAVES + w) * SCORE_RT;
    if (row0 >= n_rows)
        return;
    const int n_here = n_rows - row0 < SCORE_RT ? (int)(n_rows - row0) : SCORE_RT;
    const int n_P = G.n_P;
    double vp[SCORE_RT], vm[SCORE_RT];
    auto fetch = [&](int p0) {
        const int pi = p0 + lane;
#pragma unroll
        for (int i = 0; i < SCORE_RT; ++i) {
            vp[i] = 1.0;                  // padding: e = 0, below every real maximum
            vm[i] = 1.0;
            if (i < n_here && pi < n_P) {
                vp[i] = pred[(size_t)(row0 + i) * n_P + pi];
                vm[i] = meas[(size_t)(row0 + i) * n_P + pi];
            }
        }
    };
    fetch(0);
    // the maximum does not depend on the order: every lane keeps its own per row and the
    // lanes are combined once at the end, so that only the sum is a serial chain
    double sum = 0.0;
    double wmax[SCORE_RT];
#pragma unroll
    for (int i = 0; i < SCORE_RT; ++i)
        wmax[i] = 0.0;
    for (int p0 = 0; p0 < n_P; p0 += 64) {
#pragma unroll
        for (int i = 0; i < SCORE_RT; ++i) {
            const double err = fabs((vp[i] - vm[i]) / vm[i]);
            wmax[i] = err > wmax[i] ? err : wmax[i];
            tile[w][i][lane] = err;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (p0 + 64 < n_P)
            fetch(p0 + 64);
        if (lane < n_here) {
            const int cnt = n_P - p0 < 64 ? n_P - p0 : 64;
            int j = 0;
            for (; j + 16 <= cnt; j += 16) {           // 16 LDS reads in flight, added in order
                double err[16];
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    err[u] = tile[w][lane][j + u];
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    sum = sum + err[u];
            }
            for (; j < cnt; ++j)
                sum = sum + tile[w][lane][j];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
#pragma unroll
    for (int i = 0; i < SCORE_RT; ++i)
        tile[w][i][lane] = wmax[i];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (lane < n_here) {
        double worst = 0.0;
#pragma unroll 16
        for (int j = 0; j < 64; ++j) {
            const double v = tile[w][lane][j];
            worst = v > worst ? v : worst;
        }
        rows[2 * (row0 + lane)] = sum;
        rows[2 * (row0 + lane) + 1] = worst;
    }
}

// A wave takes one message size at a time and walks over its process counts, 64 (its lanes)
// at a time: the measured times and segment sizes of a point are fetched before any
// arithmetic (13 + 3 independent loads per lane in flight), the predictions and the verdicts
// go out, and the relative errors e = |(pred - meas) / meas| stay in the wave for the
// statistics, so that nothing is read a second time.  Per (strategy row r, m) the sum of e
// over P is one serial chain in ascending P from +0.0: the lanes leave their e in an LDS tile
// (SCORE_TILE_ROWS strategy rows at a time), then lane j adds the 64 values of row j in
// order, sixteen LDS reads at a time, and keeps the running sum for the next 64 process
// counts; the maximum does not depend on the order, every lane keeps its own per row and the
// lanes are combined once per message size.  rows[(r * n_m + mi) * 2] = {sum, max}.
// A big table is staged once per workgroup, and the waves take sizes with a stride.
constexpr int SCORE_TILE_ROWS = 7;                     // 13 strategy rows go through the tile in two halves
constexpr int SCORE_TILE_LD = 65;

// BIG: workgroups of 1024 threads (128 registers a lane); otherwise 256, and the measured times
// of the next 64 process counts are fetched while the current ones are worked on.
template <bool BIG>
__global__ void __launch_bounds__(BIG ? 1024 : 256) k_score_fused(DeviceTables T, DeviceGrid G, Scratch S,
                                                const double *__restrict__ meas,
                                                const uint32_t *__restrict__ seg,
                                                double *__restrict__ pred,
                                                plogp_verdict_dev *__restrict__ verdict,
                                                double *__restrict__ rows)
{
    extern __shared__ double lds[];
    const uint32_t mask = G.mask;
    const bool any_seg = (mask & 0x224u) != 0;
    LdsTable tab = {nullptr, nullptr, nullptr, T.n};
    if (any_seg)
        tab = stage_table(lds, T, 0);                 // for g(s) at the measured segment sizes
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n_waves = blockDim.x >> 6;
    double *tile = lds + (any_seg ? 3 * T.n : 0) + (size_t)wave * SCORE_TILE_ROWS * SCORE_TILE_LD;
    const double L = T.L[0];
    const double g1 = S.g1[0];
    const double R = __builtin_fma(3.0, L, 2.0 * g1);
    const int n_P = G.n_P;
    const size_t plane = (size_t)G.n_m * n_P;
    int n_ids = 0;
#pragma unroll
    for (int id = 0; id < 13; ++id)
        n_ids += (mask >> id) & 1u;
    auto wave_sync = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    for (int mi = blockIdx.x * n_waves + wave; mi < G.n_m; mi += gridDim.x * n_waves) {
        const u64 m = G.m[mi];
        const double gm = S.gm[mi];
        double wmax[13];                               // this lane's largest e per strategy
#pragma unroll
        for (int id = 0; id < 13; ++id)
            wmax[id] = 0.0;
        double sum_lo = 0.0, sum_hi = 0.0;             // lane j: rows j and SCORE_TILE_ROWS + j
        double tm_n[13];
        uint32_t sv_n[3] = {0u, 0u, 0u};
        auto fetch = [&](int p0, double (&tmv)[13], uint32_t (&svv)[3]) {
            const int pi = p0 + lane < n_P ? p0 + lane : n_P - 1;
            const size_t cell = (size_t)mi * n_P + pi;
            int r = 0;
#pragma unroll
            for (int id = 0; id < 13; ++id) {
                tmv[id] = 0.0;
                if ((mask >> id) & 1u) {
                    const size_t at = (size_t)r * plane + cell;
                    tmv[id] = __builtin_nontemporal_load(meas + at);
                    if (id == 2) svv[0] = seg[at];
                    if (id == 5) svv[1] = seg[at];
                    if (id == 9) svv[2] = seg[at];
                    ++r;
                }
            }
        };
        if (!BIG)
            fetch(0, tm_n, sv_n);
        for (int p0 = 0; p0 < n_P; p0 += 64) {
            const bool valid = p0 + lane < n_P;
            const int pi = valid ? p0 + lane : n_P - 1;     // padding lanes work on a valid point, quietly
            const size_t cell = (size_t)mi * n_P + pi;
            double tm[13];
            uint32_t sv[3] = {0u, 0u, 0u};
            if (BIG) {
                fetch(p0, tm, sv);
            } else {
#pragma unroll
                for (int id = 0; id < 13; ++id)
                    tm[id] = tm_n[id];
#pragma unroll
                for (int u = 0; u < 3; ++u)
                    sv[u] = sv_n[u];
                if (p0 + 64 < n_P)
                    fetch(p0 + 64, tm_n, sv_n);
            }
            const uint32_t P = G.P[pi];
            const double q = (double)(P - 1), fl = (double)floor_log2(P), cl = (double)ceil_log2(P);
            double gs[3] = {0.0, 0.0, 0.0}, k[3] = {0.0, 0.0, 0.0};
            bool ok[3] = {true, true, true};
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                if (!((mask >> (u == 0 ? 2 : u == 1 ? 5 : 9)) & 1u))
                    continue;
                const u64 sz = sv[u];
                ok[u] = sz > 0 && sz <= m;
                if (ok[u]) {
                    gs[u] = gap_at(tab, (double)sz);
                    k[u] = segments(m, sz);
                }
            }
            double best_p[2] = {INFINITY, INFINITY}, best_m[2] = {INFINITY, INFINITY};
            double meas_of_pred_best[2] = {NAN, NAN};
            uint32_t id_p[2] = {0xFFFFFFFFu, 0xFFFFFFFFu}, id_m[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};
            double ev[13];                             // e of this point per strategy (0 in padding lanes)
            int r = 0;
#pragma unroll
            for (int id = 0; id < 13; ++id) {
                ev[id] = 0.0;
                if (!((mask >> id) & 1u))
                    continue;
                const size_t at = (size_t)r * plane + cell;
                ++r;
                const double v = score_predict(id, q, fl, cl, gm, L, R, gs, k, ok, G, S, mi, pi, P);
                if (valid)
                    __builtin_nontemporal_store(v, pred + at);
                const double t_meas = tm[id];
                const double e = fabs((v - t_meas) / t_meas);
                ev[id] = valid ? e : 0.0;
                wmax[id] = ev[id] > wmax[id] ? ev[id] : wmax[id];
                const int op = id < 10 ? 0 : 1;
                if (v < best_p[op]) {
                    best_p[op] = v;
                    id_p[op] = (uint32_t)id;
                    meas_of_pred_best[op] = t_meas;
                }
                if (t_meas < best_m[op]) {
                    best_m[op] = t_meas;
                    id_m[op] = (uint32_t)id;
                }
            }
            if (valid) {
                plogp_verdict_dev *o = verdict + cell;
#pragma unroll
                for (int op = 0; op < 2; ++op) {
                    if (!(mask & (op == 0 ? 0x3FFu : 0x1C00u)))
                        continue;
                    union {
                        plogp_verdict_dev vd;
                        uint4 v;
                    } u;
                    u.vd.regret = meas_of_pred_best[op] / best_m[op] - 1.0;
                    u.vd.pred_best = id_p[op];
                    u.vd.meas_best = id_m[op];
                    stream_out(o, u.v);
                    o += plane;
                }
            }
            // the sums: the strategy rows go through the tile in two halves; a padding lane
            // holds +0.0, which leaves a sum as it is
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                int rr = 0;
#pragma unroll
                for (int id = 0; id < 13; ++id) {
                    if (!((mask >> id) & 1u))
                        continue;
                    if (rr / SCORE_TILE_ROWS == half)
                        tile[(rr % SCORE_TILE_ROWS) * SCORE_TILE_LD + lane] = ev[id];
                    ++rr;
                }
                wave_sync();
                if (half * SCORE_TILE_ROWS + lane < n_ids && lane < SCORE_TILE_ROWS) {
                    double acc = half == 0 ? sum_lo : sum_hi;
                    const double *mine = tile + lane * SCORE_TILE_LD;
#pragma unroll
                    for (int j = 0; j < 64; j += 16) {     // 16 LDS reads in flight, added in order
                        double err[16];
#pragma unroll
                        for (int u = 0; u < 16; ++u)
                            err[u] = mine[j + u];
#pragma unroll
                        for (int u = 0; u < 16; ++u)
                            acc = acc + err[u];
                    }
                    if (half == 0)
                        sum_lo = acc;
                    else
                        sum_hi = acc;
                }
                wave_sync();
            }
        }
        // the maxima over the lanes, the same way, and the two results of every row
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            int rr = 0;
#pragma unroll
            for (int id = 0; id < 13; ++id) {
                if (!((mask >> id) & 1u))
                    continue;
                if (rr / SCORE_TILE_ROWS == half)
                    tile[(rr % SCORE_TILE_ROWS) * SCORE_TILE_LD + lane] = wmax[id];
                ++rr;
            }
            wave_sync();
            const int row = half * SCORE_TILE_ROWS + lane;
            if (row < n_ids && lane < SCORE_TILE_ROWS) {
                const double *mine = tile + lane * SCORE_TILE_LD;
                double worst = 0.0;
#pragma unroll 16
                for (int j = 0; j < 64; ++j) {
                    const double v = mine[j];
                    worst = v > worst ? v : worst;
                }
                rows[2 * ((size_t)row * G.n_m + mi)] = half == 0 ? sum_lo : sum_hi;
                rows[2 * ((size_t)row * G.n_m + mi) + 1] = worst;
            }
            wave_sync();
        }
    }
}

struct plogp_score_dev {
    double sum_abs_err;
    double max_abs_err;
    unsigned long long count;
    unsigned long long reserved;
};

// Per strategy row: the per-m sums added in ascending m from +0.0.  One workgroup
// per row: 1024 per-m results are loaded side by side into LDS and thread 0 adds them
// in order while the next 1024 are in flight.
__global__ void __launch_bounds__(1024) k_score_final(DeviceGrid G, const double *rows,
                                                      plogp_score_dev *score)
{
    __shared__ double part[1024];
    __shared__ double wave_max[16];
    const int r = blockIdx.x, tid = threadIdx.x;
    const double *mine = rows + 2 * (size_t)r * G.n_m;
    double total = 0.0, worst = 0.0;        // worst: this thread's own maximum
    double a = 0.0, b = 0.0;
    if (tid < G.n_m) {
        a = mine[2 * tid];
        b = mine[2 * tid + 1];
    }
    for (int m0 = 0; m0 < G.n_m; m0 += 1024) {
        part[tid] = a;
        worst = b > worst ? b : worst;
        __syncthreads();
        const int nxt = m0 + 1024 + tid;
        b = 0.0;
        if (nxt < G.n_m) {
            a = mine[2 * (size_t)nxt];
            b = mine[2 * (size_t)nxt + 1];
        }
        if (tid == 0) {
            const int cnt = G.n_m - m0 < 1024 ? G.n_m - m0 : 1024;
            int j = 0;
            for (; j + 16 <= cnt; j += 16) {           // 16 LDS reads in flight, added in order
                double sv[16];
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    sv[u] = part[j + u];
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    total = total + sv[u];
            }
            for (; j < cnt; ++j)
                total = total + part[j];
        }
        __syncthreads();
    }
    // the maximum over all threads (any order gives the same value)
    for (int off = 32; off > 0; off >>= 1) {
        const double o = __shfl_xor(worst, off, 64);
        worst = o > worst ? o : worst;
    }
    if ((tid & 63) == 0)
        wave_max[tid >> 6] = worst;
    __syncthreads();
    if (tid == 0) {
        double top = 0.0;
        for (int i = 0; i < 16; ++i)
            top = wave_max[i] > top ? wave_max[i] : top;
        plogp_score_dev sc;
        sc.sum_abs_err = total;
        sc.max_abs_err = top;
        sc.count = (unsigned long long)G.n_m * (unsigned long long)G.n_P;
        sc.reserved = 0ull;
        score[r] = sc;
    }
}

// ---- the planes beyond Tables 1 and 2 -------------------------------------------
//
// Section 3 of the paper names Gather and Barrier as patterns that are built like
// Broadcast and Scatter.  In pLogP a Gather is its Scatter with every message
// reversed (the same sends, the other way round, over the same span of time; the
// root's receptions lie a gap apart as its sends did): rows 13..15 are the
// expressions of Table 2, on the same two sums.  A Barrier carries no payload: a
// one-byte fan-in to the root and a one-byte fan-out, flat (row 16: twice the flat
// row of Table 1 at g(1)) or binomial (row 17: twice its binomial row at g(1)); it
// does not depend on the message size.  One thread per (table, m, P), lanes along
// P; g(m), g(1) and the sums come from the staged path's first steps.
__global__ void __launch_bounds__(256) k_more_planes(DeviceTables T, DeviceGrid G, Scratch S,
                                                     plogp_cell_dev *out, int n_pchunks)
{
    int bid = (int)blockIdx.x;
    const int pi = (bid % n_pchunks) * 256 + (int)threadIdx.x;
    bid /= n_pchunks;
    const int mi = bid % G.n_m, t = bid / G.n_m;
    if (pi >= G.n_P)
        return;
    const uint32_t P = G.P[pi];
    const double L = T.L[t];
    const double q = (double)(P - 1u), fl = (double)floor_log2(P), cl = (double)ceil_log2(P);
    const size_t plane = (size_t)G.n_m * G.n_P;
    const int first = ((G.mask & 0x3FFu) ? 1 : 0) + ((G.mask & 0x1C00u) ? 1 : 0);   // planes before these
    plogp_cell_dev *o = out + ((size_t)t * G.n_ops + first) * plane + (size_t)mi * G.n_P + pi;
    if (G.extra & 7u) {
        // the rows of Table 2 under the ids of their Gather twins
        const uint32_t as_scatter = (G.extra & 7u) << 10;
        const double gm = S.gm[(size_t)t * G.n_m + mi];
        const double s11 = (as_scatter & (1u << 11)) ? chain_sum_of(G, S, t, mi, pi, P) : 0.0;
        const double s12 = (as_scatter & (1u << 12))
                               ? S.sum2[((size_t)t * G.n_m + mi) * (size_t)(G.cl_max + 1) + ceil_log2(P)] : 0.0;
        Best b = decide_scatter(as_scatter, q, cl, gm, L, s11, s12);
        b.id += 3u;
        store_cell(o, b);
        o += plane;
    }
    if (G.extra & 0x18u) {
        const double g1 = S.g1[t];
        Best b = {INFINITY, 0u, 0xFFFFFFFFu};
        if (G.extra & 8u) consider(b, 2.0 * __builtin_fma(q, g1, L), 16, 0);
        if (G.extra & 16u) consider(b, 2.0 * __builtin_fma(fl, g1, cl * L), 17, 0);
        store_cell(o, b);
    }
}

}  // namespace

// ---------------------------------------------------------------- launch wrappers

static const size_t kMaxTableLds = (size_t)3 * 4096 * sizeof(double) + 96 +
                                   (size_t)2 * SWEEP_M_MAX_S * sizeof(double);   // + g(s), 1/s in k_terms
static const size_t kMaxChainLds = (size_t)4 * 4096 * sizeof(double) + 112;   // + interval widths

static DeviceInfo g_device = {256, (size_t)160 * 1024};

const DeviceInfo &device_info() { return g_device; }

hipError_t kernels_init()
{
    hipError_t e;
    {
        int dev = 0;
        hipDeviceProp_t prop;
        if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
        if ((e = hipGetDeviceProperties(&prop, dev)) != hipSuccess) return e;
        if (prop.multiProcessorCount > 0) g_device.n_cu = prop.multiProcessorCount;
        // the kernels that fill a compute unit's LDS were laid out for 160 KB; a device that
        // reports less gets fewer workgroups per unit from the same formulas
        if (prop.maxSharedMemoryPerMultiProcessor >= (size_t)64 * 1024)
            g_device.lds_per_cu = prop.maxSharedMemoryPerMultiProcessor;
    }
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_interp),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxTableLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_eval),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxTableLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_terms),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxTableLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_chain_blocks),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxChainLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_terms_chain),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxTableLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_fused),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxTableLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_score_points),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxTableLds);
    if (e != hipSuccess) return e;
    // (the table plus the waves' tiles; the launch checks the sum against the device's LDS)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_score_fused<true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)g_device.lds_per_cu);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_score_fused<false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)g_device.lds_per_cu);
    if (e != hipSuccess) return e;
    const void *batch_kernels[4] = {
        reinterpret_cast<const void *>(k_batch_t<BATCH_T_PC, BATCH_T_PS, false, false>),
        reinterpret_cast<const void *>(k_batch_t<BATCH_T_PC, BATCH_T_PS, false, true>),
        reinterpret_cast<const void *>(k_batch_t<BATCH_T_PC, BATCH_T_PS, true, false>),
        reinterpret_cast<const void *>(k_batch_t<BATCH_T_PC, BATCH_T_PS, true, true>)};
    for (const void *k : batch_kernels) {
        e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)BATCH_T_LDS_MAX);
        if (e != hipSuccess) return e;
    }
    return e;
}

hipError_t launch_slopes(const DeviceTables &T, double *slope_out, hipStream_t st)
{
    hipLaunchKernelGGL(k_slopes, dim3(T.n_tables), dim3(256), 0, st, T, slope_out);
    return hipGetLastError();
}

hipError_t launch_interp(const DeviceTables &T, int table, const uint64_t *d_z, size_t n,
                         double *d_out, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    if ((n + 255) / 256 > 0x7FFFFFFFull) return hipErrorInvalidValue;
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
    if ((n + 255) / 256 > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const size_t lds = (size_t)3 * T.n * sizeof(double);
    const unsigned blocks = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(k_eval, dim3(blocks), dim3(256), lds, st, T, table, strategy,
                       reinterpret_cast<const u64 *>(d_m), d_P,
                       reinterpret_cast<const u64 *>(d_s), n, d_out);
    return hipGetLastError();
}

// Batches with enough (table, m) rows to fill the chip, few candidates and a short
// chain sum go through the single fused kernel; everything else through the
// staged kernels.
static bool use_fused_path(const DeviceTables &T, const DeviceGrid &G)
{
    return (long)T.n_tables * G.n_m >= 8192 && G.n_s <= FUSED_NS && G.n_blk <= 32;
}

// Few tables, few candidates, few blocks of the chain sum and many process counts: one
// workgroup per (table, m) does the whole path (k_row).
static bool use_row_path(const DeviceTables &T, const DeviceGrid &G)
{
    return G.n_s <= ROW_NS && G.n_blk <= ROW_MAX_BLK && T.n <= ROW_MAX_N && G.n_P >= 256 &&
           (long)T.n_tables * G.n_m >= 256 && (long)T.n_tables * G.n_m <= 65535 * 16;
}

// LDS of a k_batch_t workgroup: 64 tables by interval, their g(s), the output staging.
static size_t batch_t_lds(int n, int n_s)
{
    return ((size_t)2 * (n + 2) + (n_s ? n_s : 1)) * 64 * sizeof(double) +
           (size_t)BATCH_T_WAVES * BATCH_T_STAGE + (size_t)(n_s ? n_s : 1) * 4 + 16;
}

// Batches whose tables share their sample sizes, with enough tables to fill waves and
// few enough samples and candidates for the LDS staging: lanes over tables.
static bool use_table_lane_path(const DeviceTables &T, const DeviceGrid &G)
{
    // a lane's byte offset inside a store (up to 7 tables + 7 cells on) is kept in 32 bits
    const size_t table_cells = (size_t)G.n_ops * G.n_m * G.n_P;
    return T.shared_x && T.n_tables >= 64 && (long)T.n_tables * G.n_m >= 8192 &&
           table_cells <= ((size_t)1 << 24) && batch_t_lds(T.n, G.n_s) <= BATCH_T_LDS_MAX;
}

namespace {

// Lays the arrays of a plan out one after the other, each on a 256-byte boundary; the first
// 256 bytes stay free (arrays of size 0 point there).
struct LayoutBuilder {
    size_t at = 256;
    bool too_big = false;          // a size did not fit: the plan is refused
    // an array of a * b * c * d elements of `elem` bytes (a factor of 0 makes it empty)
    size_t take(size_t elem, size_t a, size_t b = 1, size_t c = 1, size_t d = 1)
    {
        constexpr size_t kMaxBytes = (size_t)1 << 46;       // no single array beyond 64 TiB: sizes stay far from wrapping
        size_t count = a;
        for (size_t f : {b, c, d}) {
            if (f != 0 && count > kMaxBytes / f) too_big = true;
            count *= f;
        }
        if (count > kMaxBytes / elem) too_big = true;
        if (too_big || count == 0) return 0;
        const size_t here = at;
        at += (count * elem + 255) & ~(size_t)255;
        return here;
    }
};

constexpr long kMaxLaunch = 0x7FFFFFFFL;      // workgroups of one launch, and int indices inside the kernels

}  // namespace

Scratch bind_scratch(void *base, const ScratchLayout &lay)
{
    char *b = static_cast<char *>(base);
    Scratch S = {};
    S.g1 = reinterpret_cast<double *>(b + lay.g1);
    S.gs = reinterpret_cast<double *>(b + lay.gs);
    S.gm = reinterpret_cast<double *>(b + lay.gm);
    S.sum2 = reinterpret_cast<double *>(b + lay.sum2);
    S.blk = reinterpret_cast<double *>(b + lay.blk);
    S.pre = reinterpret_cast<double *>(b + lay.pre);
    S.part = reinterpret_cast<double *>(b + lay.part);
    S.rcp = reinterpret_cast<double *>(b + lay.rcp);
    S.segC = reinterpret_cast<double *>(b + lay.segC);
    S.segA = reinterpret_cast<double *>(b + lay.segA);
    S.segB = reinterpret_cast<double *>(b + lay.segB);
    S.amin = reinterpret_cast<double *>(b + lay.amin);
    S.nv = reinterpret_cast<int *>(b + lay.nv);
    S.batch.rec = reinterpret_cast<double *>(b + lay.rec);
    S.batch.tab = reinterpret_cast<double *>(b + lay.tab);
    S.batch_ys = reinterpret_cast<double *>(b + lay.batch_ys);
    return S;
}

bool plan_tune(const DeviceTables &T, const DeviceGrid &G, bool terms_only, TunePlan &p)
{
    p = TunePlan{};
    p.terms_only = terms_only ? 1 : 0;
    const DeviceInfo &dev = device_info();
    const long n_cu = dev.n_cu;
    const size_t D = sizeof(double);
    const size_t nt = (size_t)T.n_tables, n_m = (size_t)G.n_m, n_mu = (size_t)G.n_mu;
    const size_t n_P = (size_t)G.n_P, n_s = (size_t)G.n_s;
    LayoutBuilder lb;
    // the rows beyond Tables 1 and 2 are formed from the staged path's terms and sums; only the
    // table-lane kernel writes their planes itself, when the Gather rows are enabled exactly as
    // the Scatter rows are (or one of the two patterns is absent): it decides once for both
    const bool fast_ok = !terms_only && G.extra == 0;
    const uint32_t scatter_rows = G.mask & 0x1C00u, gather_rows = (G.extra & 7u) << 10;
    const bool lanes_ok = !terms_only && (gather_rows == 0 || scatter_rows == 0 || gather_rows == scatter_rows);
    if (lanes_ok && use_table_lane_path(T, G)) {
        p.path = TUNE_TABLE_LANES;
        // tables by interval and the per-m facts, then everything else in one kernel
        p.n_stage = (T.n_tables + BATCH_STAGE_TT - 1) / BATCH_STAGE_TT;
        long prep_items = (long)G.n_m * (T.n + 1);
        if ((long)G.n_m * G.n_s > prep_items) prep_items = (long)G.n_m * G.n_s;
        long prep_wg = (prep_items + 255) / 256;
        if (prep_wg > 1024) prep_wg = 1024;
        p.prep_wg = (int)prep_wg;
        p.setup_lds = (size_t)BATCH_STAGE_TT * (T.n + 1) * D;
        // a workgroup: 64 tables x (BATCH_T_WAVES waves x m_per_wave sizes)
        p.n_tg = (T.n_tables + 63) / 64;
        const int per = BATCH_T_WAVES;
        int m_per_wave = 8;
        while (m_per_wave > 1 && (long)p.n_tg * ((G.n_m + per * m_per_wave - 1) / (per * m_per_wave)) < 4 * n_cu)
            m_per_wave >>= 1;
        p.m_per_wave = m_per_wave;
        p.batch_mchunks = (G.n_m + per * m_per_wave - 1) / (per * m_per_wave);
        p.batch_lds = batch_t_lds(T.n, G.n_s);
        if ((long)p.n_tg * p.batch_mchunks > kMaxLaunch) return false;
        const BatchRec R(T.n, G.n_s, G.cl_max);
        p.lay.rec = lb.take(D, n_m, (size_t)R.slots);
        p.lay.tab = lb.take(D, 2 + ((size_t)T.n + 1) + 2 * (n_s ? n_s : 1) + 4 * (size_t)batch_padded_P(G.n_P));
        p.lay.batch_ys = lb.take(D, (size_t)T.n + 2, nt, 2);
        p.lay.total = lb.at;
        return !lb.too_big;
    }
    if (fast_ok && !use_fused_path(T, G) && use_row_path(T, G)) {
        p.path = TUNE_ROW;
        // two process counts per lane when there are more groups of 64 than waves
        p.row_two = G.n_P > 64 * (ROW_THREADS / 64);
        p.row_lds = row_lds_bytes(T.n, G.n_blk, G.n_P);
        p.lay.total = lb.at;
        return true;
    }
    if (fast_ok && use_fused_path(T, G)) {
        p.path = TUNE_FUSED;
        p.fused_mchunks = (G.n_m + 255) / 256;
        if ((long)T.n_tables * p.fused_mchunks > kMaxLaunch) return false;
        p.lay.total = lb.at;
        return true;
    }
    p.path = TUNE_STAGED;
    const size_t tab_lds = (size_t)3 * T.n * D;
    // which sweep runs: lanes over s for many candidates, else lanes over P if the grid
    // has enough process counts to fill a wave, else lanes over m
    const bool lanes_s = G.n_s > SWEEP_M_MAX_S;
    const bool lanes_p = !terms_only && !lanes_s && G.n_P >= 32 && G.n_P <= 65535 * 64;   // grid.y
    // the per-(m, s) terms A, B and min_s A in device memory: only for the sweep that runs its
    // lanes over P, and only when there is a candidate at all
    const bool pairs = lanes_p && G.n_s > 0;
    p.lanes_s = lanes_s;
    p.lanes_p = lanes_p;
    p.pairs = pairs;
    long n_items = G.n_m > G.n_s ? G.n_m : G.n_s;          // a lane takes one m and one s ...
    if (pairs && (long)G.n_m * G.n_s > n_items)
        n_items = (long)G.n_m * G.n_s;                     // ... and one (m, s) pair
    long n_chunks_l = (n_items + 255) / 256;
    // the candidates go to LDS too (for the count per m) if they fit beside the table and are
    // few: every workgroup stages them all, and for 8192 of them that takes longer (11.8 us)
    // than the thirteen dependent loads of a search in device memory (6.9 us)
    const size_t pair_lds = pairs ? (size_t)2 * G.n_s * D : 0;
    const bool stage_s = G.n_s > 0 && G.n_s <= 1024 && tab_lds + pair_lds + (size_t)G.n_s * D <= kMaxTableLds;
    p.terms_mode = (pairs ? 1 : 0) | (stage_s ? 2 : 0);
    p.terms_lds = tab_lds + pair_lds + (stage_s ? (size_t)G.n_s * D : 0);
    // a workgroup stages the whole table: with a big table one workgroup fits a CU, so no
    // more workgroups than CUs
    const long wg_cap = p.terms_lds > 65536 ? n_cu : 2 * n_cu;
    const long chunk_cap = wg_cap / T.n_tables > 1 ? wg_cap / T.n_tables : 1;
    if (n_chunks_l > chunk_cap) n_chunks_l = chunk_cap;
    // the per-size part in workgroups of its own, beside the others: freely for small tables;
    // for a big table (one workgroup per CU) out of the same budget of workgroups
    int n_mchunks = 0;
    if (p.terms_lds <= 16384) {
        n_mchunks = ((G.n_m + 63) / 64 + 3) / 4;
        const int cap = n_cu / T.n_tables > 1 ? (int)(n_cu / T.n_tables) : 1;
        if (n_mchunks > cap) n_mchunks = cap;
    } else if (T.n_tables == 1 && n_chunks_l >= 64) {
        n_mchunks = ((G.n_m + 63) / 64 + 3) / 4;
        if (n_mchunks > n_chunks_l / 8) n_mchunks = (int)(n_chunks_l / 8);
        if (n_chunks_l + n_mchunks > chunk_cap) n_chunks_l = chunk_cap - n_mchunks;
    }
    p.n_chunks = (int)n_chunks_l;
    p.n_mchunks = n_mchunks;
    const long terms_wg = (long)T.n_tables * (p.n_chunks + n_mchunks);
    if (terms_wg > kMaxLaunch) return false;
    p.terms_wg = (int)terms_wg;
    const bool chain = (G.need & (1u << 11)) != 0;
    p.chain = chain;
    // a big table fills most of the LDS of a CU: one large workgroup per CU then, which
    // stays for its whole share of the work (the table is staged once)
    p.chain_lds = (size_t)4 * T.n * D + 112;
    const bool big = p.chain_lds > 32768;
    // few samples, few blocks, enough distinct sizes: a workgroup per (table, m) forms all
    // its sums, the prefix over the blocks included
    p.crow_lds = chain_row_lds(T.n, G.n_blk);
    p.chain_row = chain && T.n <= 512 && G.n_blk <= CROW_MAX_BLK && p.crow_lds <= 65536 &&
                  (long)T.n_tables * G.n_mu >= 128 && (long)T.n_tables * G.n_mu <= (1L << 24);
    // small tables: the terms and the chain sums in one launch, side by side
    p.together = chain && !big && !p.chain_row;
    // (terms beside the per-row chain sums: when the terms need little LDS)
    p.row_together = p.chain_row && p.terms_lds <= 65536;
    // a big table: the workgroups of the chain sums do the terms when they run out of sums
    p.terms_in_chain = chain && big && !p.chain_row && p.terms_lds <= p.chain_lds;
    if (p.chain_row) {
        if ((long)p.terms_wg + (long)T.n_tables * G.n_mu > kMaxLaunch) return false;
    } else if (chain) {
        p.chain_threads = big ? 1024 : 256;
        const int n_mg = (G.n_mu + 63) / 64;
        // leading blocks that are items of their own: the dense part of a table with many
        // samples (its first blocks search per term), or every block when the whole sum is
        // too small to fill the chip with units of CHAIN_U blocks
        int n_single = T.n > 256 ? 32 : 0, n_search = T.n > 256 ? 4 : 0;
        if ((long)T.n_tables * n_mg * ((G.n_blk + CHAIN_U - 1) / CHAIN_U) < 8 * n_cu) n_single = G.n_blk;
        if (n_single > G.n_blk) n_single = G.n_blk;
        if (n_search > n_single) n_search = n_single;
        const long items = (long)n_mg * (n_single + (G.n_blk - n_single + CHAIN_U - 1) / CHAIN_U);
        if (items > kMaxLaunch) return false;
        long wg = (big ? n_cu : 4 * n_cu) / T.n_tables;
        const long wg_need = (items + p.chain_threads / 64 - 1) / (p.chain_threads / 64);
        if (wg > wg_need) wg = wg_need;
        if (wg < 1) wg = 1;
        // a small job (the walk would be bound by one lane's latency): every term by a search
        const double n_terms = (double)T.n_tables * G.n_mu * G.n_blk * SUM_BLOCK;
        const bool small = p.together && n_single == G.n_blk && n_terms <= (double)(3L << 20);
        p.both_lds = p.chain_lds > p.terms_lds ? p.chain_lds : p.terms_lds;
        if (small) {
            const size_t small_lds = ((size_t)3 * T.n + 10 + 64 * SMALL_LD) * D;
            if (small_lds > p.both_lds) p.both_lds = small_lds;
            n_single = -1;
            wg = (long)n_mg * G.n_blk;
            // the chain workgroups come first in the grid: they must leave the terms
            // workgroups room on the chip, or those would only start when these are done
            long room = n_cu * (long)(dev.lds_per_cu / (p.both_lds + 512)) - (long)p.terms_wg;
            if (room > 2 * n_cu) room = 2 * n_cu;
            if (wg > room / T.n_tables) wg = room / T.n_tables;
            if (wg < 1) wg = 1;
        }
        p.n_single = n_single;
        p.n_search = n_search;
        p.chain_wg = (int)wg;
        if ((long)T.n_tables * wg + p.terms_wg > kMaxLaunch) return false;
        p.n_chain_wg = (int)(T.n_tables * wg);
        p.n_mgroups = (G.n_mu + PFX_M - 1) / PFX_M;
        if ((long)T.n_tables * p.n_mgroups > kMaxLaunch) return false;
    }
    if (!terms_only) {
        if (lanes_s) {
            // 8 waves per workgroup (two per SIMD, so that two workgroups share a CU); the
            // process counts per wave are chosen so that one workgroup covers all of them if
            // it can
            const int waves = SWEEP_S_MAX_WAVES;
            p.sweep_gp = G.n_P <= 6 * waves ? 6 : (G.n_P <= 9 * waves ? 9 : 12);
            p.sweep_ptiles = p.sweep_gp == 12 ? (G.n_P + 12 * waves - 1) / (12 * waves) : 1;
            if ((long)T.n_tables * G.n_m * p.sweep_ptiles > kMaxLaunch) return false;
        } else if (lanes_p) {
            // as many waves as the chip holds at four per SIMD, shared out over the tables and
            // the groups of 64 process counts; each walks over every n_w-th message size;
            // two process counts per lane when the grid has at least 512 of them
            const bool all = G.mask == 0x1FFFu;
            p.ppl = G.n_P >= 512 && G.n_s <= 64 && all ? 2 : 1;
            p.n_pg = (G.n_P + 64 * p.ppl - 1) / (64 * p.ppl);
            // (a big job - 6 x 4096 groups of cells - runs best with one size per wave:
            // 33.5 us against 37.8 with six)
            const long wave_budget = (long)T.n_tables * p.n_pg * G.n_m >= 64 * n_cu ? 256 * n_cu * p.ppl : 32 * n_cu;
            long n_w = wave_budget / p.ppl / ((long)T.n_tables * p.n_pg);
            if (n_w > G.n_m) n_w = G.n_m;
            if (n_w < 1) n_w = 1;
            n_w = (n_w + 3) / 4 * 4;
            p.n_w = (int)n_w;
        } else {
            constexpr int PC = 4;
            p.n_mg = (G.n_m + 63) / 64;
            p.n_pcg = (G.n_P + 4 * PC - 1) / (4 * PC);
            if ((long)T.n_tables * p.n_mg * p.n_pcg > kMaxLaunch) return false;
        }
    }
    if (!terms_only && G.extra != 0 && (long)T.n_tables * G.n_m * ((G.n_P + 255) / 256) > kMaxLaunch) return false;
    // scratch: what the kernels of this path index (m-fastest arrays per distinct size where noted)
    const bool binom = (G.need & (1u << 12)) != 0;
    p.lay.g1 = lb.take(D, nt);
    p.lay.gs = lb.take(D, nt, n_s);
    p.lay.gm = lb.take(D, nt, n_m);
    p.lay.sum2 = lb.take(D, binom ? nt : 0, n_m, (size_t)(G.cl_max + 1));
    p.lay.blk = lb.take(D, chain ? nt : 0, (size_t)G.n_blk, n_mu);
    p.lay.part = lb.take(D, chain ? nt : 0, n_mu, n_P);
    p.lay.pre = lb.take(D, chain && G.blk_is_prefix ? nt : 0, n_mu, n_P);
    p.lay.rcp = lb.take(D, n_s);
    p.lay.segC = lb.take(D, nt, n_s);
    p.lay.segA = lb.take(D, pairs ? nt : 0, n_m, n_s);
    p.lay.segB = lb.take(D, pairs ? nt : 0, n_m, n_s);
    p.lay.amin = lb.take(D, pairs ? nt : 0, n_m);
    p.lay.nv = lb.take(sizeof(int), n_m);
    if (terms_only)
        p.lay.score_rows = lb.take(D, 13, n_m, 2);
    p.lay.total = lb.at;
    return !lb.too_big;
}

hipError_t launch_tune_stage(const TunePlan &p, int stage, const DeviceTables &T, const DeviceGrid &G,
                             const Scratch &S, plogp_cell_dev *d_out, hipStream_t st)
{
    if (p.path == TUNE_TABLE_LANES) {
        if (stage == TUNE_STAGE_TERMS) {
            hipLaunchKernelGGL(k_batch_setup, dim3((unsigned)(p.n_stage + p.prep_wg)), dim3(256), p.setup_lds,
                               st, T, G, S.batch, reinterpret_cast<f64x2 *>(S.batch_ys), p.n_stage);
        } else if (stage == TUNE_STAGE_SWEEP) {
            BatchDims D;
            D.n = T.n; D.n_tables = T.n_tables; D.n_m = G.n_m; D.n_P = G.n_P; D.n_s = G.n_s;
            D.cl_max = G.cl_max; D.n_ops = G.n_ops; D.n_mchunks = p.batch_mchunks; D.m_per_wave = p.m_per_wave;
            D.mask = G.mask;
            D.extra = G.extra;
            const bool all = G.mask == 0x1FFFu, more = G.extra != 0;
            const auto kern = all ? (more ? k_batch_t<BATCH_T_PC, BATCH_T_PS, true, true>
                                          : k_batch_t<BATCH_T_PC, BATCH_T_PS, true, false>)
                                  : (more ? k_batch_t<BATCH_T_PC, BATCH_T_PS, false, true>
                                          : k_batch_t<BATCH_T_PC, BATCH_T_PS, false, false>);
            hipLaunchKernelGGL(kern, dim3((unsigned)p.n_tg * p.batch_mchunks), dim3(64 * BATCH_T_WAVES),
                               p.batch_lds, st, D, reinterpret_cast<const f64x2 *>(S.batch_ys), T.L,
                               S.batch.rec, S.batch.tab, reinterpret_cast<const u64 *>(G.s), d_out);
        }
        return hipGetLastError();
    }
    if (p.path == TUNE_ROW) {
        if (stage == TUNE_STAGE_SWEEP) {
            const bool all = G.mask == 0x1FFFu, two = p.row_two != 0;
            const auto kern = all ? (two ? k_row<true, 2> : k_row<true, 1>) : (two ? k_row<false, 2> : k_row<false, 1>);
            hipLaunchKernelGGL(kern, dim3((unsigned)(T.n_tables * G.n_m)), dim3(ROW_THREADS), p.row_lds, st,
                               T, G, d_out);
        }
        return hipGetLastError();
    }
    if (p.path == TUNE_FUSED) {
        if (stage == TUNE_STAGE_SWEEP)
            hipLaunchKernelGGL(k_fused, dim3((unsigned)T.n_tables * p.fused_mchunks), dim3(256),
                               (size_t)3 * T.n * sizeof(double) + 64, st, T, G, d_out, p.fused_mchunks);
        return hipGetLastError();
    }
    if (stage == TUNE_STAGE_MORE) {
        if (!p.terms_only && G.extra != 0) {
            const int n_pchunks = (G.n_P + 255) / 256;
            hipLaunchKernelGGL(k_more_planes, dim3((unsigned)((long)T.n_tables * G.n_m * n_pchunks)), dim3(256), 0,
                               st, T, G, S, d_out, n_pchunks);
        }
        return hipGetLastError();
    }
    switch (stage) {
    case TUNE_STAGE_TERMS:
        if (!p.together && !p.row_together && !p.terms_in_chain)
            hipLaunchKernelGGL(k_terms, dim3((unsigned)p.terms_wg), dim3(256), p.terms_lds, st, T, G, S,
                               p.n_chunks, p.n_mchunks, p.terms_mode);
        break;
    case TUNE_STAGE_CHAIN:
        if (p.chain_row) {
            if (p.row_together)
                hipLaunchKernelGGL(k_terms_chain_row, dim3((unsigned)(p.terms_wg + T.n_tables * G.n_mu)),
                                   dim3(CROW_THREADS), p.crow_lds > p.terms_lds ? p.crow_lds : p.terms_lds, st,
                                   T, G, S, p.terms_wg, p.n_chunks, p.n_mchunks, p.terms_mode);
            else
                hipLaunchKernelGGL(k_chain_row, dim3((unsigned)(T.n_tables * G.n_mu)), dim3(CROW_THREADS),
                                   p.crow_lds, st, T, G, S);
        } else if (p.chain) {
            if (p.together)
                hipLaunchKernelGGL(k_terms_chain, dim3((unsigned)(p.n_chain_wg + p.terms_wg)), dim3(256),
                                   p.both_lds, st, T, G, S, p.n_chain_wg, p.chain_wg, p.n_single, p.n_search,
                                   p.n_chunks, p.n_mchunks, p.terms_mode);
            else
                hipLaunchKernelGGL(k_chain_blocks, dim3((unsigned)p.n_chain_wg), dim3(p.chain_threads),
                                   p.chain_lds, st, T, G, S, p.chain_wg, p.n_single, p.n_search,
                                   p.terms_in_chain ? p.terms_mode : -1);
        }
        break;
    case TUNE_STAGE_PREFIX:
        if (p.chain && !p.chain_row && G.blk_is_prefix)
            hipLaunchKernelGGL(k_chain_prefix, dim3((unsigned)T.n_tables * p.n_mgroups), dim3(256), 0, st, G, S,
                               p.n_mgroups);
        break;
    default:
        if (p.terms_only)
            break;
        if (p.lanes_s) {
            const unsigned rows = (unsigned)T.n_tables * G.n_m;
            const dim3 threads(64 * SWEEP_S_MAX_WAVES);
            if (p.sweep_gp == 6)
                hipLaunchKernelGGL(k_sweep_s<6>, dim3(rows), threads, 0, st, T, G, S, d_out, 1);
            else if (p.sweep_gp == 9)
                hipLaunchKernelGGL(k_sweep_s<9>, dim3(rows), threads, 0, st, T, G, S, d_out, 1);
            else
                hipLaunchKernelGGL(k_sweep_s<12>, dim3(rows * p.sweep_ptiles), threads, 0, st, T, G, S, d_out,
                                   p.sweep_ptiles);
        } else if (p.lanes_p) {
            const bool all = G.mask == 0x1FFFu;
            for (int t0 = 0; t0 < T.n_tables; t0 += 65535) {
                const int nt = T.n_tables - t0 < 65535 ? T.n_tables - t0 : 65535;
                const dim3 blocks((unsigned)(p.n_w / 4), (unsigned)p.n_pg, (unsigned)nt);
                if (G.n_s <= 64 && all && p.ppl == 2)
                    hipLaunchKernelGGL((k_sweep_p<1, true, 2>), blocks, dim3(256), 0, st, T, G, S, d_out, t0, p.n_w);
                else if (G.n_s <= 64 && all)
                    hipLaunchKernelGGL((k_sweep_p<1, true, 1>), blocks, dim3(256), 0, st, T, G, S, d_out, t0, p.n_w);
                else if (G.n_s <= 64)
                    hipLaunchKernelGGL((k_sweep_p<1, false, 1>), blocks, dim3(256), 0, st, T, G, S, d_out, t0, p.n_w);
                else
                    hipLaunchKernelGGL((k_sweep_p<4, false, 1>), blocks, dim3(256), 0, st, T, G, S, d_out, t0, p.n_w);
            }
        } else {
            hipLaunchKernelGGL(k_sweep_m<4>, dim3((unsigned)T.n_tables * p.n_mg * p.n_pcg), dim3(256), 0, st, T, G,
                               S, d_out, p.n_mg, p.n_pcg);
        }
        break;
    }
    return hipGetLastError();
}

hipError_t launch_score_stage(int stage, const TunePlan &plan, const DeviceTables &T1, const DeviceGrid &G,
                              const Scratch &S, double *rows, const double *d_meas, const uint32_t *d_seg,
                              double *d_pred, void *d_verdict, void *d_scores, hipStream_t st)
{
    int n_ids = 0;
    for (int id = 0; id < 13; ++id) n_ids += (G.mask >> id) & 1u;
    if (stage == 0)      // g(m), g(1), the Scatter sums: the first stages of the tuning
        return launch_tune(plan, T1, G, S, nullptr, st);
    // With many message sizes a wave takes a whole size and forms the error sums on the way
    // (one pass over the measurements); with fewer there would be too few waves to hide the
    // memory latency of their serial walks, and the points go one to a thread with the sums
    // formed by a second pass.
    const bool fused = G.n_m >= 8 * device_info().n_cu;
    const size_t tab_lds = (G.mask & 0x224u) ? (size_t)3 * T1.n * sizeof(double) : 0;
    // a small table is staged by every workgroup of 256; a big one by as few workgroups of 1024
    // as fill the compute units, which then walk their items with a stride
    const bool big = tab_lds > 16384;
    const int threads = big ? 1024 : 256;
    const DeviceInfo &dev = device_info();
    if (stage == 1 && fused) {
        const int waves = threads / 64;
        const size_t lds = tab_lds + (size_t)waves * SCORE_TILE_ROWS * SCORE_TILE_LD * sizeof(double);
        if (lds > dev.lds_per_cu) return hipErrorInvalidValue;
        long n_wg = ((long)G.n_m + waves - 1) / waves;
        if (big) {
            const long fit = (long)dev.n_cu * (long)(dev.lds_per_cu / lds);
            if (n_wg > fit) n_wg = fit;
        }
        hipLaunchKernelGGL(big ? k_score_fused<true> : k_score_fused<false>, dim3((unsigned)n_wg), dim3(threads),
                           lds, st, T1, G, S, d_meas, d_seg, d_pred,
                           reinterpret_cast<plogp_verdict_dev *>(d_verdict), rows);
        return hipGetLastError();
    }
    if (stage == 1) {
        const int n_pchunks = (G.n_P + threads - 1) / threads;
        const long n_items = (long)G.n_m * n_pchunks;
        long n_wg = n_items;
        if (big) {
            const long fit = (long)dev.n_cu * (long)(dev.lds_per_cu / tab_lds);
            if (n_wg > fit) n_wg = fit;
        }
        if (n_items > kMaxLaunch) return hipErrorInvalidValue;
        hipLaunchKernelGGL(k_score_points, dim3((unsigned)n_wg), dim3(threads), tab_lds, st, T1, G, S, d_meas,
                           d_seg, d_pred, reinterpret_cast<plogp_verdict_dev *>(d_verdict), n_pchunks,
                           (int)n_items);
        return hipGetLastError();
    }
    if (!fused) {
        const long n_rows = (long)n_ids * G.n_m;
        const long row_wg = (n_rows + SCORE_RT * SCORE_WAVES - 1) / (SCORE_RT * SCORE_WAVES);
        hipLaunchKernelGGL(k_score_rows, dim3((unsigned)row_wg), dim3(64 * SCORE_WAVES), 0, st, G, n_ids, d_meas,
                           d_pred, rows);
    }
    // the per-m sums of every strategy added in ascending m
    hipLaunchKernelGGL(k_score_final, dim3((unsigned)n_ids), dim3(1024), 0, st, G, rows,
                       reinterpret_cast<plogp_score_dev *>(d_scores));
    return hipGetLastError();
}

}  // namespace plogp
