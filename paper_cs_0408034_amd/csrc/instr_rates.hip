// Issue cost of a few gfx950 instructions, measured: every lane runs a loop of eight
// independent instructions of one kind (or one dependent chain), with 8 or 1 workgroups of
// 4 waves per CU; HIP events time the second of two launches.  Timing only, no memory
// traffic beyond one store per lane.  Not part of the library:
//   hipcc --offload-arch=gfx950 -O3 -o /tmp/instr_rates paper_cs_0408034_amd/csrc/instr_rates.hip
//   /tmp/instr_rates
#include <hip/hip_runtime.h>
#include <cstdio>
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("hip error %d at %s:%d\n", (int)e, __FILE__, __LINE__); return 1; } } while (0)

template <int OP>
__global__ void __launch_bounds__(256) k(double *out, int iters, double a, double b)
{
    double v[8];
    for (int i = 0; i < 8; ++i) v[i] = a + threadIdx.x * 1e-9 + i;
    double c = b;
    int sc = iters;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (OP == 0) asm volatile("v_fma_f64 %0, %0, %1, %2" : "+v"(v[i]) : "v"(c), "v"(a));
            if (OP == 1) asm volatile("v_min_f64 %0, %0, %1" : "+v"(v[i]) : "v"(c));
            if (OP == 2) asm volatile("v_add_f64 %0, %0, %1" : "+v"(v[i]) : "v"(c));
            if (OP == 3) asm volatile("v_max_f64 %0, %0, %1" : "+v"(v[i]) : "v"(c));
            if (OP == 4) asm volatile("v_mul_f64 %0, %0, %1" : "+v"(v[i]) : "v"(c));
            if (OP == 5) asm volatile("v_cmp_lt_f64 vcc, %0, %1" : : "v"(v[i]), "v"(c) : "vcc");
            if (OP == 6) asm volatile("v_add_f32 %0, %0, %1" : "+v"(*(float *)&v[i]) : "v"((float)1.0f));
            if (OP == 8) asm volatile("v_mov_b32 %0, %1" : "=v"(*(int *)&v[i]) : "v"(it));
            if (OP == 9) asm volatile("v_fma_f64 %0, %0, %1, %2" : "+v"(v[0]) : "v"(c), "v"(a));       // one dependent chain
            if (OP == 10) asm volatile("v_add_u32 %0, %0, %1" : "+v"(*(int *)&v[i]) : "v"(3));
            if (OP == 11) asm volatile("s_add_u32 %0, %0, 1" : "+s"(sc) : : "scc");
            if (OP == 12) asm volatile("v_min_f64 %0, %0, %1" : "+v"(v[0]) : "v"(c));                   // dependent min
        }
    }
    double s = 0;
    for (int i = 0; i < 8; ++i) s += v[i];
    s += sc;
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int OP>
int run(const char *name, double *d, int per_cu = 8)
{
    const int blocks = 256 * per_cu, iters = 4096;      // 8 workgroups of 4 waves per CU: 8 waves per SIMD
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    hipLaunchKernelGGL(k<OP>, dim3(blocks), dim3(256), 0, 0, d, iters, 1.0, 1.0000001);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0, 0));
    hipLaunchKernelGGL(k<OP>, dim3(blocks), dim3(256), 0, 0, d, iters, 1.0, 1.0000001);
    CHECK(hipEventRecord(e1, 0));
    CHECK(hipEventSynchronize(e1));
    float ms = 0;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    // wave instructions per SIMD: blocks * 4 waves / 1024 SIMDs * iters * 8
    const double per_simd = (double)blocks * 4 / 1024.0 * iters * 8;
    const double cycles = ms * 1e-3 * 2.4e9;
    printf("%-14s (%d wg/cu) %.3f ms  %.2f cycles per wave instruction (at 2.4 GHz)\n", name, per_cu, ms, cycles / per_simd);
    fflush(stdout);
    return 0;
}

int main()
{
    double *d;
    CHECK(hipMalloc(&d, (size_t)256 * 8 * 256 * sizeof(double)));
    if (run<0>("v_fma_f64", d)) return 1;
    if (run<1>("v_min_f64", d)) return 1;
    if (run<2>("v_add_f64", d)) return 1;
    if (run<3>("v_max_f64", d)) return 1;
    if (run<4>("v_mul_f64", d)) return 1;
    if (run<5>("v_cmp_lt_f64", d)) return 1;
    if (run<6>("v_add_f32", d)) return 1;
    if (run<8>("v_mov_b32", d)) return 1;
    if (run<10>("v_add_u32", d)) return 1;
    if (run<11>("s_add_u32", d)) return 1;
    if (run<9>("fma dependent", d)) return 1;
    if (run<9>("fma dependent", d, 1)) return 1;
    if (run<0>("v_fma_f64", d, 1)) return 1;
    if (run<6>("v_add_f32", d, 1)) return 1;
    if (run<12>("min dependent", d)) return 1;
    CHECK(hipFree(d));
    return 0;
}
