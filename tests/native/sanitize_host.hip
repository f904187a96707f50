// Driver for a sanitizer pass over the HOST code of the library (argument validation, grid
// preparation, the launch plan and its scratch layout), built with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host side only.  Runs with or without a GPU: without one
// every compute entry point must stop at PLOGP_EDEVICE after its host-side work.
#include "../../include/plogp.h"
#include "../../include/plogp_profile.h"
#include "../../paper_cs_0408034_amd/csrc/plogp_internal.hpp"

#include <cstdio>
#include <cstdlib>
#include <vector>

static unsigned long long state = 0x243F6A8885A308D3ull;
static unsigned long long next_u64()
{
    unsigned long long z = (state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static int pick(int lo, int hi) { return lo + (int)(next_u64() % (unsigned long long)(hi - lo + 1)); }

#define CHECK(cond)                                                            \
    do {                                                                       \
        if (!(cond)) { std::printf("check failed at line %d: %s\n", __LINE__, #cond); return 1; } \
    } while (0)

int main()
{
    // ---- the C ABI: refused arguments, then valid ones (PLOGP_OK with a GPU, PLOGP_EDEVICE without)
    plogp_table *tab = nullptr;
    plogp_grid *grid = nullptr;
    const double x[4] = {1.0, 8.0, 64.0, 4096.0}, y[4] = {3.0, 3.5, 5.0, 40.0}, ybad[4] = {3.0, -1.0, 5.0, 40.0};
    CHECK(plogp_load_table(nullptr, y, 4, 1.0, &tab) == PLOGP_EINVAL);
    CHECK(plogp_load_table(x, ybad, 4, 1.0, &tab) == PLOGP_EINVAL);
    CHECK(plogp_load_table(x, y, 1, 1.0, &tab) == PLOGP_EINVAL);
    const int st_tab = plogp_load_table(x, y, 4, 7.25, &tab);
    CHECK(st_tab == PLOGP_OK || st_tab == PLOGP_EDEVICE);
    std::vector<uint64_t> m, s;
    std::vector<uint32_t> P;
    for (int i = 0; i < 300; ++i) m.push_back(8ull * (1 + next_u64() % 100000));
    for (int i = 0; i < 40; ++i) m.push_back(m[i]);                     // repeats
    for (uint32_t p = 2; p < 3000; p += 1 + p / 7) P.push_back(p);
    for (uint64_t v = 8; v <= (1u << 20); v *= 2) s.push_back(v);
    plogp_grid_desc d = {m.data(), m.size(), P.data(), P.size(), s.data(), s.size(), PLOGP_NO_CAP, 8, PLOGP_MASK_EVERY};
    const int st_grid = plogp_grid_create(&d, &grid);
    CHECK(st_grid == PLOGP_OK || st_grid == PLOGP_EDEVICE);
    plogp_grid_desc bad = d;
    bad.strategy_mask = 1u << 18;
    CHECK(plogp_grid_create(&bad, &grid) == PLOGP_EINVAL);
    bad = d;
    bad.n_P = 0;
    CHECK(plogp_grid_create(&bad, &grid) == PLOGP_EINVAL);
    std::vector<uint64_t> big = {1ull << 40};
    std::vector<uint32_t> bigP = {2, 1u << 14};
    plogp_grid_desc rng = {big.data(), 1, bigP.data(), 2, s.data(), s.size(), PLOGP_NO_CAP, 8, PLOGP_MASK_ALL};
    CHECK(plogp_grid_create(&rng, &grid) == PLOGP_ERANGE);
    CHECK(plogp_tune_grid(nullptr, nullptr, nullptr, 0, nullptr) == PLOGP_EINVAL);
    CHECK(plogp_tune_grid_static(nullptr, nullptr, nullptr, 0, nullptr) == PLOGP_EINVAL);
    float ms5[5];
    CHECK(plogp_tune_grid_profile(nullptr, nullptr, nullptr, 0, nullptr, 1, ms5) == PLOGP_EINVAL);
    CHECK(plogp_decision_table_bytes(3, nullptr) == 0);
    if (st_tab == PLOGP_OK && st_grid == PLOGP_OK) {
        CHECK(plogp_grid_ops(grid) == 4);
        CHECK(plogp_decision_table_bytes(1, grid) == 4 * m.size() * P.size() * 16);
        plogp_grid_free(grid);
        plogp_free_table(tab);
    }

    // ---- the launch plan and its scratch layout over many shapes (host arithmetic only)
    long plans = 0;
    for (int it = 0; it < 20000; ++it) {
        plogp::DeviceTables T = {};
        plogp::DeviceGrid G = {};
        const int nts[] = {1, 1, 2, 5, 64, 100, 10000, 1 << 20};
        const int nsam[] = {2, 21, 64, 512, 1100, 4096};
        T.n_tables = nts[pick(0, 7)];
        T.n = nsam[pick(0, 5)];
        T.shared_x = pick(0, 1);
        G.n_m = pick(0, 3) == 0 ? pick(1, 1 << 24) : pick(1, 5000);
        G.n_mu = pick(1, G.n_m);
        G.n_P = pick(0, 3) == 0 ? pick(1, 1 << 20) : pick(1, 1200);
        G.n_s = pick(0, 4) == 0 ? 0 : (pick(0, 3) == 0 ? pick(1, 1 << 16) : pick(1, 300));
        const int p_top = 1 << (pick(0, 1) ? 24 : 12);
        const unsigned Pmax = (unsigned)pick(G.n_P + 1, p_top > G.n_P + 1 ? p_top : G.n_P + 1);
        G.n_blk = (int)((Pmax - 1) / 64) + 1;
        G.last_terms = (int)((Pmax - 1) - 64u * (unsigned)(G.n_blk - 1));
        G.cl_max = 0;
        while ((1u << G.cl_max) < Pmax) ++G.cl_max;
        const unsigned mask = (unsigned)pick(1, PLOGP_MASK_EVERY);
        G.mask = mask & PLOGP_MASK_ALL;
        G.extra = mask >> 13;
        G.need = (((mask >> 11) | (mask >> 14)) & 1u) << 11 | (((mask >> 12) | (mask >> 15)) & 1u) << 12;
        G.n_ops = ((mask & 0x3FFu) != 0) + ((mask & 0x1C00u) != 0) + ((mask & 0xE000u) != 0) + ((mask & 0x30000u) != 0);
        G.blk_is_prefix = G.n_blk > 32;
        for (int terms_only = 0; terms_only < 2; ++terms_only) {
            plogp::TunePlan plan;
            if (!plogp::plan_tune(T, G, terms_only != 0, plan))
                continue;                                        // too large for one launch: refused, not wrapped
            ++plans;
            const plogp::ScratchLayout &l = plan.lay;
            const size_t offs[] = {l.g1, l.gs, l.gm, l.sum2, l.blk, l.pre, l.part, l.rcp, l.segC, l.segA, l.segB,
                                   l.amin, l.nv, l.rec, l.tab, l.batch_ys, l.score_rows};
            for (size_t o : offs)
                CHECK(o < l.total && o % 256 == 0);
            CHECK(plan.path >= 0 && plan.path <= 3);
            // rows beyond the tables: the staged path, or the table-lane kernel when the Gather
            // rows are enabled exactly as the Scatter rows are (or one of the two is absent)
            const unsigned scatter_rows = G.mask & 0x1C00u, gather_rows = (G.extra & 7u) << 10;
            const bool lanes_may = gather_rows == 0 || scatter_rows == 0 || gather_rows == scatter_rows;
            if (terms_only)
                CHECK(plan.path == plogp::TUNE_STAGED);
            else if (G.extra != 0)
                CHECK(plan.path == plogp::TUNE_STAGED || (plan.path == plogp::TUNE_TABLE_LANES && lanes_may));
            if (plan.path == plogp::TUNE_STAGED && plan.pairs)
                CHECK(l.segA != 0 && l.segB != 0 && l.amin != 0 && G.n_s > 0);
        }
    }
    std::printf("host sanitizer pass: %ld plans laid out\n", plans);
    return 0;
}
