/* Driver for a sanitizer pass over the CPU oracle: builds small tables and grids with a
 * fixed generator and calls every entry point of oracle/plogp_oracle.c (compiled into this
 * program with -fsanitize=address,undefined), including empty candidate lists, one-sample
 * tails, P at block boundaries and every strategy id.  Prints a checksum; any finding of the
 * sanitizers aborts the run. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct { double time; uint32_t s; uint32_t strategy; } cell;
typedef struct { double regret; uint32_t pred_best; uint32_t meas_best; } verdict;
typedef struct { double sum_abs_err; double max_abs_err; uint64_t count; uint64_t reserved; } score;

void plogp_oracle_slopes(const double *x, const double *y, size_t n, double *slope);
double plogp_oracle_g(const double *x, const double *y, size_t n, double z);
int plogp_oracle_eval(const double *x, const double *y, size_t n, double L, int id, uint64_t m, uint32_t P,
                      uint64_t s, double *out);
int plogp_oracle_tune(const double *x, const double *y, size_t n, const double *L, size_t n_tables,
                      const uint64_t *m, size_t n_m, const uint32_t *P, size_t n_P, const uint64_t *s,
                      size_t n_s, uint64_t s_cap, uint32_t mask, cell *out, int n_threads);
int plogp_oracle_score(const double *x, const double *y, size_t n, double L, const uint64_t *m, size_t n_m,
                       const uint32_t *P, size_t n_P, uint32_t mask, const double *meas, const uint32_t *seg,
                       double *pred, verdict *v, score *sc);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint64_t next(void)
{
    uint64_t z = (state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

int main(void)
{
    double sum = 0.0;
    const size_t ns[] = {2, 3, 64, 257};
    for (size_t ni = 0; ni < 4; ++ni) {
        const size_t n = ns[ni], n_tables = 3;
        double *x = malloc(n_tables * n * sizeof(double)), *y = malloc(n_tables * n * sizeof(double));
        double L[3] = {0.0, 55.0, 7.25};
        for (size_t t = 0; t < n_tables; ++t) {
            double at = 1.0 + (double)(next() % 16);
            for (size_t i = 0; i < n; ++i) {
                x[t * n + i] = at;
                y[t * n + i] = 3.0 + at / 11.5 * (1.0 + (double)(next() % 100) / 1000.0);
                at += 1.0 + (double)(next() % 5000);
            }
        }
        const uint64_t m[] = {8, 8, 64, 4096, 4104, 1 << 20, (1ull << 30) + 8};
        const uint32_t P[] = {2, 3, 64, 65, 66, 129, 1000, 4097};
        const uint64_t s[] = {8, 24, 64, 4096, 1 << 16};
        const size_t n_m = 7, n_P = 8;
        const uint32_t masks[] = {0x3FFFF, 0x1FFF, 0x3FF, 0x1C00, 0xE000, 0x30000, 1u << 5, (1u << 14) | (1u << 2)};
        for (size_t mk = 0; mk < 8; ++mk) {
            for (size_t n_s = 0; n_s <= 5; n_s += 5) {
                int ops = 0;
                const uint32_t op_mask[4] = {0x3FF, 0x1C00, 0xE000, 0x30000};
                for (int o = 0; o < 4; ++o) ops += (masks[mk] & op_mask[o]) != 0;
                cell *out = malloc(n_tables * (size_t)ops * n_m * n_P * sizeof(cell));
                if (plogp_oracle_tune(x, y, n, L, n_tables, m, n_m, P, n_P, s, n_s, mk % 2 ? 4096 : UINT64_MAX,
                                      masks[mk], out, 2) < 0)
                    return 2;
                for (size_t i = 0; i < n_tables * (size_t)ops * n_m * n_P; ++i)
                    if (isfinite(out[i].time)) sum += out[i].time + out[i].s + out[i].strategy;
                free(out);
            }
        }
        for (int id = 0; id < 18; ++id) {
            double v;
            if (plogp_oracle_eval(x, y, n, 55.0, id, 4104, 66, 24, &v) != 0) return 3;
            sum += v;
            if (plogp_oracle_eval(x, y, n, 55.0, id, 0, 66, 24, &v) != -1) return 4;       /* refused: m = 0 */
        }
        if (plogp_oracle_eval(x, y, n, 55.0, 18, 8, 2, 8, &sum) != -1) return 5;           /* unknown id */
        sum += plogp_oracle_g(x, y, n, 1.0) + plogp_oracle_g(x, y, n, 9007199254740991.0);
        /* scoring on the same grid */
        const uint32_t mask = 0x1FFF;
        const size_t rows = 13;
        double *meas = malloc(rows * n_m * n_P * sizeof(double)), *pred = malloc(rows * n_m * n_P * sizeof(double));
        uint32_t *seg = malloc(rows * n_m * n_P * sizeof(uint32_t));
        for (size_t r = 0; r < rows; ++r)
            for (size_t mi = 0; mi < n_m; ++mi)
                for (size_t pi = 0; pi < n_P; ++pi) {
                    meas[(r * n_m + mi) * n_P + pi] = 10.0 + (double)(next() % 100000);
                    seg[(r * n_m + mi) * n_P + pi] = 8;
                }
        verdict *ver = malloc(2 * n_m * n_P * sizeof(verdict));
        score sc[13];
        if (plogp_oracle_score(x, y, n, 55.0, m, n_m, P, n_P, mask, meas, seg, pred, ver, sc) != 0) return 6;
        for (size_t r = 0; r < rows; ++r) sum += sc[r].sum_abs_err;
        free(meas); free(pred); free(seg); free(ver); free(x); free(y);
    }
    printf("oracle sanitizer pass: checksum %.17g\n", sum);
    return 0;
}
