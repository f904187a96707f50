// Write bandwidth of decision-table store patterns on gfx950, measured: a wave holds the
// cells of 64 tables and writes RUN neighbouring cells (16 bytes each) of one table with RUN
// neighbouring lanes, so a store instruction covers 64 / RUN tables whose rows lie one
// whole table apart.  Shape of the batched workload: 157 x 64 tables x 2 operations x
// 256 sizes x 24 process counts (1.98 GB).  HIP events, best of three launches.  Timing
// only, values are arbitrary.  Also a contiguous fill under each store cache policy.
// Not part of the library:
//   hipcc --offload-arch=gfx950 -O3 -o /tmp/store_patterns paper_cs_0408034_amd/csrc/store_patterns.hip
//   /tmp/store_patterns
#include <hip/hip_runtime.h>
#include <cstdio>
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("hip error %d at %s:%d\n", (int)e, __FILE__, __LINE__); return 1; } } while (0)

constexpr int N_OPS = 2, N_M = 256, N_P = 24, N_TG = 157, WAVES = 16;
constexpr size_t TABLE_CELLS = (size_t)N_OPS * N_M * N_P;
constexpr size_t TOTAL_CELLS = (size_t)N_TG * 64 * TABLE_CELLS;

// RUN cells of one table are written together by RUN neighbouring lanes; a store instruction
// covers 64 / RUN tables, RUN... instructions cover the 64 tables of the wave.
template <int RUN>
__global__ void __launch_bounds__(64 * WAVES) k_runs(uint4 *out, int n_mchunks, int m_per_wave, int lds_pad)
{
    extern __shared__ uint4 lds[];
    const int tg = blockIdx.x / n_mchunks, mc = blockIdx.x % n_mchunks;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int RPI = 64 / RUN;                    // runs per instruction
    const int r = lane / RUN, c = lane % RUN;
    const bool active = r < RPI;
    if (lds_pad) lds[threadIdx.x] = make_uint4(0, 0, 0, 0);
    for (int mw = 0; mw < m_per_wave; ++mw) {
        const int mi = (mc * WAVES + wave) * m_per_wave + mw;
        if (mi >= N_M) break;
        for (int op = 0; op < N_OPS; ++op)
            for (int p0 = 0; p0 < N_P; p0 += RUN) {
                if (!active || p0 + c >= N_P) continue;
                for (int tb = 0; tb < 64; tb += RPI) {
                    const int table = tb + r;
                    if (table >= 64) break;
                    const size_t cell = ((size_t)tg * 64 + table) * TABLE_CELLS + (size_t)op * N_M * N_P + (size_t)mi * N_P + p0 + c;
                    out[cell] = make_uint4(mi, op, p0 + c, table);
                }
            }
    }
}

__global__ void __launch_bounds__(1024) k_contig(uint4 *out, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        out[i] = make_uint4((unsigned)i, 1, 2, 3);
}

template <int RUN>
int run(uint4 *d, int m_per_wave, size_t lds_bytes)
{
    const int n_mchunks = (N_M + WAVES * m_per_wave - 1) / (WAVES * m_per_wave);
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(k_runs<RUN>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    float best = 1e30f;
    for (int rep = 0; rep < 4; ++rep) {
        CHECK(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(k_runs<RUN>, dim3(N_TG * n_mchunks), dim3(64 * WAVES), lds_bytes, 0, d, n_mchunks, m_per_wave, lds_bytes ? 1 : 0);
        CHECK(hipGetLastError());
        CHECK(hipEventRecord(e1, 0));
        CHECK(hipEventSynchronize(e1));
        float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
        if (rep > 0 && ms < best) best = ms;
    }
    printf("runs of %2d cells (%4d B), m_per_wave %d, lds %6zu: %.3f ms  %.0f GB/s\n", RUN, RUN * 16, m_per_wave, lds_bytes, best,
           TOTAL_CELLS * 16.0 / best * 1e-6);
    fflush(stdout);
    return 0;
}

template <int POL>
__global__ void __launch_bounds__(1024) k_contig_pol(uint4 *out, size_t n)
{
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        u32x4 v = {(unsigned)i, 1u, 2u, 3u};
        uint4 *p = out + i;
        if (POL == 0) asm volatile("global_store_dwordx4 %0, %1, off" : : "v"(p), "v"(v) : "memory");
        if (POL == 1) asm volatile("global_store_dwordx4 %0, %1, off nt" : : "v"(p), "v"(v) : "memory");
        if (POL == 2) asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" : : "v"(p), "v"(v) : "memory");
        if (POL == 3) asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
        if (POL == 4) asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt" : : "v"(p), "v"(v) : "memory");
    }
}

template <int POL>
int run_pol(uint4 *d, const char *name)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    float best = 1e30f;
    for (int rep = 0; rep < 4; ++rep) {
        CHECK(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(k_contig_pol<POL>, dim3(4096), dim3(1024), 0, 0, d, TOTAL_CELLS);
        CHECK(hipGetLastError());
        CHECK(hipEventRecord(e1, 0));
        CHECK(hipEventSynchronize(e1));
        float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
        if (rep > 0 && ms < best) best = ms;
    }
    printf("contiguous, policy %-12s: %.3f ms  %.0f GB/s\n", name, best, TOTAL_CELLS * 16.0 / best * 1e-6);
    fflush(stdout);
    return 0;
}

int main()
{
    uint4 *d;
    CHECK(hipMalloc((void **)&d, TOTAL_CELLS * 16));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    for (int blocks : {1024, 4096}) {
        float best = 1e30f;
        for (int rep = 0; rep < 4; ++rep) {
            CHECK(hipEventRecord(e0, 0));
            hipLaunchKernelGGL(k_contig, dim3(blocks), dim3(1024), 0, 0, d, TOTAL_CELLS);
            CHECK(hipGetLastError());
            CHECK(hipEventRecord(e1, 0));
            CHECK(hipEventSynchronize(e1));
            float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
            if (rep > 0 && ms < best) best = ms;
        }
        printf("contiguous, %d blocks: %.3f ms  %.0f GB/s\n", blocks, best, TOTAL_CELLS * 16.0 / best * 1e-6);
        fflush(stdout);
    }
    if (run_pol<0>(d, "default")) return 1;
    if (run_pol<1>(d, "nt")) return 1;
    if (run_pol<2>(d, "sc0 sc1")) return 1;
    if (run_pol<3>(d, "sc1")) return 1;
    if (run_pol<4>(d, "sc0 sc1 nt")) return 1;
    for (size_t lds : {(size_t)0, (size_t)150 * 1024}) {     // 150 KB: one workgroup per CU, as in the library
        for (int mpw : {2, 8}) {
            if (run<4>(d, mpw, lds)) return 1;
            if (run<8>(d, mpw, lds)) return 1;
            if (run<12>(d, mpw, lds)) return 1;
            if (run<24>(d, mpw, lds)) return 1;
        }
    }
    CHECK(hipFree(d));
    return 0;
}
