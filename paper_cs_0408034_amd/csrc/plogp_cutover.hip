// gfx950 kernels of the cut-over extraction: each row (table, operation, P)
// of a decision table, read along the message sizes, is compressed into its
// runs of equal decision.  This is the form in which the tuned decisions are
// applied (paper, Section 3.1: above some message size a collective is
// segmented, below it is not; Section 1: one technique per pattern, message
// size and node count).
//
// Integer and index work only; the result is unique, so it must equal the
// plain definition bit for bit.
//
// Three steps, all bound by HBM traffic:
//   k_cut_mark  one thread per (row, tile of CUT_TM sizes): compares the key of
//               every cell with the key of the cell before it, keeps the start
//               flags of the tile as a bit mask and their count;
//   k_cut_scan1 / k_cut_scan2  exclusive prefix of the counts in (row, tile)
//               order: per workgroup of CUT_SCAN_WG counts, then over the
//               workgroup totals;
//   k_cut_emit  one thread per (row, tile) again: writes a run record for every
//               flagged cell at its place, and the row offsets.
// The decision table is stored [table][operation][m][P] with P fastest, so the
// lanes of a wave run over consecutive P (coalesced) and, when the grid has
// fewer than 64 process counts, over consecutive tiles as well.
//
// Tables of many rows and at most CUT_ROWS_MAX_M sizes take one pass instead
// (k_cut_rows): a thread owns a whole row, so a workgroup of 256 consecutive
// rows owns a contiguous stretch of the output; it reads its rows once, keeps
// the start flags in registers, learns where its stretch begins from the
// workgroups before it (their totals, published through one 64-bit word each)
// and writes its runs - the table is read once, nothing else goes through
// device memory.
#include "plogp_internal.hpp"

namespace plogp {
namespace {

typedef unsigned long long u64;

struct CutShape {
    int n_tables, n_ops, n_m, n_P;
    int n_tiles;      // tiles of CUT_TM sizes per row
    int lp;           // lanes of a wave along P: a power of two, at most 64
    int n_pg;         // groups of lp process counts
    long n_items;     // n_tables * n_ops * n_pg * n_tiles * lp threads
};

// Thread -> (row, tile).  Returns false for the padding lanes past n_P.
__device__ __forceinline__ bool cut_item(const CutShape &sh, long item, int &t, int &op, int &pi,
                                         int &tile)
{
    const int pl = (int)(item % sh.lp);
    item /= sh.lp;
    tile = (int)(item % sh.n_tiles);
    item /= sh.n_tiles;
    const int pg = (int)(item % sh.n_pg);
    item /= sh.n_pg;
    op = (int)(item % sh.n_ops);
    t = (int)(item / sh.n_ops);
    pi = pg * sh.lp + pl;
    return pi < sh.n_P;
}

// (s, strategy) of a cell: the second half of its 16-byte record.  STREAM: the table is far
// larger than the caches and every record is read once, so the loads carry the non-temporal
// hint (3 % off the pass over a 2 GB table; on a table that fits the caches the hint costs 24 %).
template <bool STREAM>
__device__ __forceinline__ uint2 cell_key(const plogp_cell_dev *cells, size_t idx)
{
    if (STREAM) {
        typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
        const u32x2_t k = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t *>(cells) + idx * 2 + 1);
        return make_uint2(k.x, k.y);
    }
    return reinterpret_cast<const uint2 *>(cells)[idx * 2 + 1];
}

template <bool STREAM>
__global__ void __launch_bounds__(256) k_cut_mark(CutShape sh, const plogp_cell_dev *cells, int key_mode,
                                                  uint32_t *counts, uint32_t *flags)
{
    const long item = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (item >= sh.n_items)
        return;
    int t, op, pi, tile;
    if (!cut_item(sh, item, t, op, pi, tile))
        return;
    const int m0 = tile * CUT_TM;
    const int len = sh.n_m - m0 < CUT_TM ? sh.n_m - m0 : CUT_TM;
    const size_t base = ((size_t)(t * sh.n_ops + op) * sh.n_m + m0) * sh.n_P + pi;
    // all keys of the tile and the one before it are fetched before any is compared
    uint2 key[CUT_TM + 1];
    key[0] = m0 > 0 ? cell_key<STREAM>(cells, base - sh.n_P) : make_uint2(0u, 0u);
#pragma unroll
    for (int k = 0; k < CUT_TM; ++k)
        key[k + 1] = k < len ? cell_key<STREAM>(cells, base + (size_t)k * sh.n_P) : make_uint2(0u, 0u);
    uint32_t bits = 0u;
#pragma unroll
    for (int k = 0; k < CUT_TM; ++k) {
        bool differs = key[k + 1].y != key[k].y;              // strategy
        if (key_mode == 1)
            differs = differs || key[k + 1].x != key[k].x;    // and segment size
        if (k < len && (differs || (m0 == 0 && k == 0)))      // the first cell of a row starts a run
            bits |= 1u << k;
    }
    const size_t row = (size_t)(t * sh.n_ops + op) * sh.n_P + pi;
    counts[row * sh.n_tiles + tile] = (uint32_t)__builtin_popcount(bits);
    flags[row * sh.n_tiles + tile] = bits;
}

// Exclusive prefix inside each group of CUT_SCAN_WG counts and the group
// totals.  A thread takes CUT_SCAN_PER consecutive counts.
__global__ void __launch_bounds__(CUT_SCAN_THREADS) k_cut_scan1(const uint32_t *counts, uint32_t *local,
                                                                 size_t n, u64 *group_total)
{
    __shared__ uint32_t wave_sum[CUT_SCAN_THREADS / 64];
    const size_t first = ((size_t)blockIdx.x * CUT_SCAN_THREADS + threadIdx.x) * CUT_SCAN_PER;
    uint32_t v[CUT_SCAN_PER];
    uint32_t sum = 0u;
#pragma unroll
    for (int k = 0; k < CUT_SCAN_PER; ++k) {
        v[k] = first + k < n ? counts[first + k] : 0u;
        sum += v[k];
    }
    // inclusive scan of the thread sums over the wave (log steps through the lanes)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t up = (uint32_t)__shfl_up((int)inc, d, 64);
        if (lane >= d)
            inc += up;
    }
    if (lane == 63)
        wave_sum[wave] = inc;
    __syncthreads();
    uint32_t before = 0u, total = 0u;
#pragma unroll
    for (int w = 0; w < CUT_SCAN_THREADS / 64; ++w) {
        before += w < wave ? wave_sum[w] : 0u;
        total += wave_sum[w];
    }
    uint32_t run = before + inc - sum;
#pragma unroll
    for (int k = 0; k < CUT_SCAN_PER; ++k) {
        if (first + k < n)
            local[first + k] = run;
        run += v[k];
    }
    if (threadIdx.x == 0)
        group_total[blockIdx.x] = total;
}

// Exclusive prefix of the group totals (in place), one workgroup; the grand
// total goes to *total_out (the entry after the last row offset).
__global__ void __launch_bounds__(1024) k_cut_scan2(u64 *group_total, size_t n_groups, u64 *total_out)
{
    __shared__ u64 wave_sum[16];
    __shared__ u64 carry_s;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0)
        carry_s = 0ull;
    __syncthreads();
    for (size_t g0 = 0; g0 < n_groups; g0 += 1024) {
        const size_t i = g0 + threadIdx.x;
        const u64 v = i < n_groups ? group_total[i] : 0ull;
        u64 inc = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const u64 up = (u64)__shfl_up((long long)inc, d, 64);
            if (lane >= d)
                inc += up;
        }
        if (lane == 63)
            wave_sum[wave] = inc;
        __syncthreads();
        u64 before = carry_s, all = 0ull;
        for (int w = 0; w < 16; ++w) {
            before += w < wave ? wave_sum[w] : 0ull;
            all += wave_sum[w];
        }
        if (i < n_groups)
            group_total[i] = before + inc - v;
        __syncthreads();
        if (threadIdx.x == 0)
            carry_s += all;
        __syncthreads();
    }
    if (threadIdx.x == 0)
        *total_out = carry_s;
}

struct plogp_run_dev {
    u64 m_from;
    uint32_t s;
    uint32_t strategy;
};

// n_fused > 0: group_before still holds the n_fused (at most CUT_FUSE_MAX) group totals; every
// workgroup forms their exclusive prefix itself in LDS, workgroup 0 also writes the grand
// total to *total_out - one launch fewer for the small jobs, which are bound by launches.
constexpr int CUT_FUSE_MAX = 1024;

__global__ void __launch_bounds__(256) k_cut_emit(CutShape sh, const plogp_cell_dev *cells, const u64 *m,
                                                  const uint32_t *local, const uint32_t *flags,
                                                  const u64 *group_before, u64 *row_offsets,
                                                  plogp_run_dev *runs, u64 capacity, int n_fused,
                                                  u64 *total_out)
{
    __shared__ u64 gpre[CUT_FUSE_MAX];
    __shared__ u64 wsum[4];
    if (n_fused > 0) {
        // four totals per thread, in order; scan over the wave, then over the four waves
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        u64 v[4], sum = 0ull;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int g = (int)threadIdx.x * 4 + k;
            v[k] = g < n_fused ? group_before[g] : 0ull;
            sum += v[k];
        }
        u64 inc = sum;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const u64 up = (u64)__shfl_up((long long)inc, d, 64);
            if (lane >= d)
                inc += up;
        }
        if (lane == 63)
            wsum[wave] = inc;
        __syncthreads();
        u64 before = 0ull, all = 0ull;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            before += w < wave ? wsum[w] : 0ull;
            all += wsum[w];
        }
        u64 run = before + inc - sum;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            gpre[threadIdx.x * 4 + k] = run;
            run += v[k];
        }
        if (blockIdx.x == 0 && threadIdx.x == 0)
            *total_out = all;
        __syncthreads();
    }
    const long item = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (item >= sh.n_items)
        return;
    int t, op, pi, tile;
    if (!cut_item(sh, item, t, op, pi, tile))
        return;
    const size_t row = (size_t)(t * sh.n_ops + op) * sh.n_P + pi;
    const size_t idx = row * sh.n_tiles + tile;
    u64 at = (n_fused > 0 ? gpre[idx / CUT_SCAN_WG] : group_before[idx / CUT_SCAN_WG]) + local[idx];
    if (tile == 0)
        row_offsets[row] = at;
    uint32_t bits = flags[idx];
    const int m0 = tile * CUT_TM;
    const size_t base = ((size_t)(t * sh.n_ops + op) * sh.n_m + m0) * sh.n_P + pi;
    while (bits != 0u) {
        const int k = __builtin_ctz(bits);
        bits &= bits - 1u;
        if (at < capacity) {
            const uint2 key = cell_key<false>(cells, base + (size_t)k * sh.n_P);
            union {
                plogp_run_dev r;
                uint4 v;
            } u;
            u.r.m_from = m[m0 + k];
            u.r.s = key.x;
            u.r.strategy = key.y;
            reinterpret_cast<uint4 *>(runs)[at] = u.v;
        }
        ++at;
    }
}

// ---- one pass, a thread per row ------------------------------------------------
//
// ctl[0]: the next workgroup number (workgroups number themselves in the order in
// which they start, so that every lower number belongs to a workgroup that is
// running or done); ctl[1]: set if a wait was given up; ctl[2 + w]: the status of
// workgroup w, one word that carries its state in the two top bits (0 nothing
// yet, 1 the number of runs of its rows, 2 the number of runs of all rows up to
// and including its own) and the count in the others.  The words are written and
// read with device-scope atomics: value and state travel together, so no other
// ordering is needed.  A workgroup publishes state 1 before it waits for anyone,
// and waits only for lower numbers: every wait ends.  The waits are bounded all
// the same (spin_limit polls): a workgroup that gives up sets ctl[1] and goes on
// with a wrong offset rather than hold the device.
constexpr unsigned long long CUT_STATE_SHIFT = 62, CUT_COUNT_MASK = (1ull << 62) - 1ull;

__global__ void __launch_bounds__(256) k_cut_rows_clear(u64 *ctl, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n)
        ctl[i] = 0ull;
}

__device__ __forceinline__ u64 wave_sum_u64(u64 v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1)
        v += (u64)__shfl_xor((long long)v, d, 64);
    return v;
}

// NW: 32-bit words of start flags per row (the grid has at most 32 NW sizes).
template <bool STREAM, int NW>
__global__ void __launch_bounds__(256) k_cut_rows(CutShape sh, const plogp_cell_dev *cells, const u64 *m,
                                                  int key_mode, u64 *ctl, u64 *row_offsets,
                                                  plogp_run_dev *runs, u64 capacity, u64 n_rows,
                                                  unsigned spin_limit)
{
    __shared__ unsigned wg_s;
    __shared__ u64 wave_total[4];
    __shared__ u64 before_s;
    __shared__ uint2 kept[CUT_ROWS_KEEP][256];         // the keys of a row's first run starts
    if (threadIdx.x == 0)
        wg_s = (unsigned)atomicAdd(ctl, 1ull);
    __syncthreads();
    const unsigned wg = wg_s;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u64 row = (u64)wg * 256 + threadIdx.x;
    const bool live = row < n_rows;
    const u64 rr = live ? row : n_rows - 1;            // padding threads read a valid row
    const u64 plane = rr / (u64)sh.n_P;                // table * n_ops + operation
    const int pi = (int)(rr % (u64)sh.n_P);
    const size_t base = (size_t)plane * sh.n_m * sh.n_P + pi;

    // first pass over the row: where a run starts
    uint32_t bits[NW];
    uint2 prev = make_uint2(0u, 0u);
    int starts = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        bits[w] = 0u;
        if (32 * w >= sh.n_m)
            continue;                                  // the same for every thread
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int m0 = 32 * w + 16 * half;
            uint2 key[16];                             // sixteen keys are fetched before any is compared
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const int mi = m0 + k < sh.n_m ? m0 + k : sh.n_m - 1;
                key[k] = cell_key<STREAM>(cells, base + (size_t)mi * sh.n_P);
            }
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                bool differs = key[k].y != prev.y;
                if (key_mode == 1)
                    differs = differs || key[k].x != prev.x;
                if (m0 + k < sh.n_m && (differs || m0 + k == 0)) {
                    bits[w] |= 1u << (16 * half + k);
                    if (starts < CUT_ROWS_KEEP)
                        kept[starts][threadIdx.x] = key[k];
                    ++starts;
                }
                prev = key[k];
            }
        }
    }
    u64 count = live ? (u64)starts : 0ull;

    // the runs before this row: inside the workgroup by a scan, before the workgroup from
    // the status words of the lower-numbered workgroups
    u64 inc = count;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const u64 up = (u64)__shfl_up((long long)inc, d, 64);
        if (lane >= d)
            inc += up;
    }
    if (lane == 63)
        wave_total[wave] = inc;
    __syncthreads();
    u64 inside = inc - count, total = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        inside += w < wave ? wave_total[w] : 0ull;
        total += wave_total[w];
    }
    if (wave == 0) {
        u64 before = 0;
        if (wg > 0) {
            if (lane == 0)
                __hip_atomic_store(ctl + 2 + wg, (1ull << CUT_STATE_SHIFT) | total, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            long long j = (long long)wg - 1;           // the nearest workgroup not yet counted
            unsigned polls = 0;
            for (;;) {
                // 64 status words at a time, lane l looks at workgroup j - l
                const long long idx = j - lane;
                u64 sv = 2ull << CUT_STATE_SHIFT;      // before workgroup 0: nothing, and final
                if (idx >= 0)
                    sv = __hip_atomic_load(ctl + 2 + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const u64 state = sv >> CUT_STATE_SHIFT;
                const u64 known = __ballot(state != 0ull), final_ = __ballot(state == 2ull);
                const int stop = final_ ? __builtin_ctzll(final_) : 63;      // counted up to this lane
                const u64 wanted = (2ull << stop) - 1ull;                    // lanes 0 .. stop
                if ((known & wanted) == wanted) {
                    before += wave_sum_u64(lane <= stop ? (sv & CUT_COUNT_MASK) : 0ull);
                    if (final_)
                        break;
                    j -= 64;
                    continue;
                }
                if (++polls > spin_limit) {
                    if (lane == 0)
                        atomicExch(ctl + 1, 1ull);
                    break;
                }
                __builtin_amdgcn_s_sleep(4);
            }
        }
        if (lane == 0) {
            __hip_atomic_store(ctl + 2 + wg, (2ull << CUT_STATE_SHIFT) | (before + total), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            before_s = before;
        }
    }
    __syncthreads();
    u64 at = before_s + inside;
    if (!live)
        return;
    row_offsets[row] = at;
    if (row == n_rows - 1)
        row_offsets[n_rows] = at + count;              // the grand total
    // second pass: a record per start flag; the keys of the first few were kept, those of the
    // others are read once more
    int nth = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        uint32_t b = bits[w];
        while (b != 0u) {
            const int k = 32 * w + __builtin_ctz(b);
            b &= b - 1u;
            const int mine = nth++;
            if (at < capacity) {
                const uint2 key = mine < CUT_ROWS_KEEP ? kept[mine][threadIdx.x]
                                                       : cell_key<false>(cells, base + (size_t)k * sh.n_P);
                union {
                    plogp_run_dev r;
                    uint4 v;
                } u;
                u.r.m_from = m[k];
                u.r.s = key.x;
                u.r.strategy = key.y;
                reinterpret_cast<uint4 *>(runs)[at] = u.v;
            }
            ++at;
        }
    }
}

}  // namespace

bool cutover_by_rows(const DeviceGrid &G, int n_tables)
{
    // enough rows to fill the chip with one thread each, and few enough sizes for the start
    // flags of a row to stay in registers
    const size_t n_rows = (size_t)n_tables * G.n_ops * G.n_P;
    return G.n_m <= CUT_ROWS_MAX_M && n_rows >= (size_t)128 * device_info().n_cu;
}

size_t cutover_ctl_words(const DeviceGrid &G, int n_tables)
{
    const size_t n_rows = (size_t)n_tables * G.n_ops * G.n_P;
    return (n_rows + 255) / 256 + 2;
}

size_t cutover_items(const DeviceGrid &G, int n_tables)
{
    const size_t n_tiles = ((size_t)G.n_m + CUT_TM - 1) / CUT_TM;
    return (size_t)n_tables * G.n_ops * G.n_P * n_tiles;
}

hipError_t launch_cutovers_stage(int stage, const DeviceGrid &G, int n_tables, const plogp_cell_dev *d_cells,
                                 int key_mode, const CutScratch &C, uint64_t *d_row_offsets, void *d_runs,
                                 uint64_t capacity, hipStream_t st)
{
    CutShape sh;
    sh.n_tables = n_tables;
    sh.n_ops = G.n_ops;
    sh.n_m = G.n_m;
    sh.n_P = G.n_P;
    sh.n_tiles = (G.n_m + CUT_TM - 1) / CUT_TM;
    int lp = 1;
    while (lp < 64 && lp < G.n_P) lp <<= 1;
    sh.lp = lp;
    sh.n_pg = (G.n_P + lp - 1) / lp;
    sh.n_items = (long)n_tables * G.n_ops * sh.n_pg * sh.n_tiles * lp;
    const size_t n_counts = cutover_items(G, n_tables);
    const size_t n_groups = (n_counts + CUT_SCAN_WG - 1) / CUT_SCAN_WG;
    const size_t n_rows = (size_t)n_tables * G.n_ops * G.n_P;
    // one thread per (row, tile), padded to whole waves along P: must fit one launch
    if ((sh.n_items + 255) / 256 > 0x7FFFFFFFL || n_groups > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const unsigned blocks = (unsigned)((sh.n_items + 255) / 256);
    const bool fuse = n_groups <= (size_t)CUT_FUSE_MAX;     // the prefix of the group totals inside the last step
    if (cutover_by_rows(G, n_tables)) {
        // one pass, a thread per row (stage 0; the other stages have nothing to do)
        if (stage != 0) return hipSuccess;
        const size_t n_wg = (n_rows + 255) / 256;
        if (n_wg > 0x7FFFFFFFull) return hipErrorInvalidValue;
        u64 *ctl = reinterpret_cast<u64 *>(C.ctl);
        hipLaunchKernelGGL(k_cut_rows_clear, dim3((unsigned)((n_wg + 2 + 255) / 256)), dim3(256), 0, st, ctl,
                           n_wg + 2);
        const bool stream = (size_t)n_rows * G.n_m * sizeof(plogp_cell_dev) > ((size_t)256 << 20);
        const bool wide = G.n_m > 32 * 8;
        const auto kern = stream ? (wide ? k_cut_rows<true, 16> : k_cut_rows<true, 8>)
                                 : (wide ? k_cut_rows<false, 16> : k_cut_rows<false, 8>);
        hipLaunchKernelGGL(kern, dim3((unsigned)n_wg), dim3(256), 0, st, sh, d_cells,
                           reinterpret_cast<const u64 *>(G.m), key_mode, ctl,
                           reinterpret_cast<u64 *>(d_row_offsets), reinterpret_cast<plogp_run_dev *>(d_runs),
                           (u64)capacity, (u64)n_rows, CUT_SPIN_LIMIT);
        return hipGetLastError();
    }
    if (stage == 0) {
        // a table beyond the 256 MB of the last-level cache is streamed
        const bool stream = n_counts * CUT_TM * sizeof(plogp_cell_dev) > ((size_t)256 << 20);
        hipLaunchKernelGGL(stream ? k_cut_mark<true> : k_cut_mark<false>, dim3(blocks), dim3(256), 0, st, sh,
                           d_cells, key_mode, C.counts, C.flags);
    } else if (stage == 1) {
        hipLaunchKernelGGL(k_cut_scan1, dim3((unsigned)n_groups), dim3(CUT_SCAN_THREADS), 0, st,
                           C.counts, C.local, n_counts, reinterpret_cast<u64 *>(C.group_total));
        if (!fuse)
            hipLaunchKernelGGL(k_cut_scan2, dim3(1), dim3(1024), 0, st,
                               reinterpret_cast<u64 *>(C.group_total), n_groups,
                               reinterpret_cast<u64 *>(d_row_offsets) + n_rows);
    } else {
        hipLaunchKernelGGL(k_cut_emit, dim3(blocks), dim3(256), 0, st, sh, d_cells,
                           reinterpret_cast<const u64 *>(G.m), C.local, C.flags,
                           reinterpret_cast<const u64 *>(C.group_total),
                           reinterpret_cast<u64 *>(d_row_offsets),
                           reinterpret_cast<plogp_run_dev *>(d_runs), (u64)capacity, fuse ? (int)n_groups : 0,
                           reinterpret_cast<u64 *>(d_row_offsets) + n_rows);
    }
    return hipGetLastError();
}

}  // namespace plogp
