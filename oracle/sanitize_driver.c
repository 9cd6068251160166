/* Drives every entry point of ozaki_oracle.c on exactly sized heap buffers, for a build with
 * -fsanitize=address,undefined (tests/test_sanitizers.py): an access outside a buffer, a shift out of range,
 * a signed overflow or an out-of-range float-to-int conversion anywhere in the oracle stops the run.
 * TEST INFRASTRUCTURE ONLY, like the oracle itself.  Inputs: a small fixed 64-bit generator (the numbers do
 * not matter, their spread does): values (u - 0.5) exp(phi z) plus planted zeros, powers of two, subnormals
 * and huge magnitudes. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oz_beta(int64_t n);
int64_t oz_r(int64_t n, int beta);
int64_t oz_count_addends(int k, int64_t r);
void oz_row_exponents(int64_t m, int64_t n, const double *A, int32_t *eA);
void oz_col_exponents(int64_t n, int64_t p, const double *B, int32_t *eB);
void oz_exponents_floor(int64_t rows, int64_t cols_, const double *X, int by_col, int32_t *e);
void oz_split_rows(int64_t m, int64_t n, const double *A, const int32_t *eA, int beta, int k, int form, int8_t *SA);
void oz_split_cols(int64_t n, int64_t p, const double *B, const int32_t *eB, int beta, int k, int form, int8_t *SB);
void oz_split_per_slice(int64_t rows, int64_t cols_, const double *X, int by_col, int beta, int k, int form,
                        int8_t *S, int32_t *E);
int64_t oz_group_chunk(int64_t m, int64_t n, int64_t p, const int8_t *SA, const int8_t *SB, int g, int s0, int s1,
                       int32_t *C);
void oz_accumulate(int64_t m, int64_t p, const int32_t *C, const int32_t *eA, const int32_t *eB, int beta, int g,
                   int first, double *D);
int64_t oz_r_wide(int64_t n, int beta);
int64_t oz_dgemm_variant(int64_t m, int64_t n, int64_t p, const double *A, const double *B, int k, int split_mode,
                         int r_mode, double *D, int64_t *n_addends);
int64_t oz_dgemm_per_slice(int64_t m, int64_t n, int64_t p, const double *A, const double *B, int k, double *D,
                           int64_t *n_addends);
int64_t oz_dgemm(int64_t m, int64_t n, int64_t p, const double *A, const double *B, int k, double *D,
                 int64_t *n_addends);
void oz_dot2_gemm(int64_t m, int64_t n, int64_t p, const double *A, const double *B, double *Rhi, double *Rlo);
int oz_num_threads(void);
void oz_axpby(int64_t m, int64_t p, double alpha, const double *D, double beta, double *C);

static uint64_t state = 0x9e3779b97f4a7c15ull;
static double uniform01(void)
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (double)(state >> 11) * (1.0 / 9007199254740992.0);
}
static double normal01(void)
{
    double u = uniform01(), v = uniform01();
    if (u < 1e-300) u = 1e-300;
    return sqrt(-2.0 * log(u)) * cos(6.283185307179586 * v);
}

static double *matrix(int64_t rows, int64_t cols, double phi, int plant)
{
    double *x = (double *)malloc((size_t)(rows * cols > 0 ? rows * cols : 1) * sizeof(double));
    for (int64_t i = 0; i < rows * cols; ++i) x[i] = (uniform01() - 0.5) * exp(phi * normal01());
    if (plant && rows * cols >= 8) {
        x[0] = 0.0;
        x[1] = 1.0;
        x[2] = -0.5;
        x[3] = 4.9406564584124654e-324; /* smallest subnormal */
        x[4] = -2.2250738585072014e-308;
        x[5] = ldexp(1.0, 900);
        x[6] = -ldexp(1.0, 900) * 1.9999999999999998;
        x[7] = 3.0;
    }
    return x;
}

static int run_case(int64_t m, int64_t n, int64_t p, int k, double phi, int plant)
{
    int beta = oz_beta(n > 0 ? n : 1);
    double *A = matrix(m, n, phi, plant), *B = matrix(n, p, phi, plant);
    double *D = (double *)malloc((size_t)(m * p > 0 ? m * p : 1) * sizeof(double));
    double *D2 = (double *)malloc((size_t)(m * p > 0 ? m * p : 1) * sizeof(double));
    int64_t w = 0, bad = 0;
    /* whole-path entry points */
    bad += oz_dgemm(m, n, p, A, B, k, D, &w);
    for (int split = 0; split < 2; ++split)
        for (int rm = 0; rm < 3; ++rm) {
            if (rm == 2 && split != 0) continue;
            bad += oz_dgemm_variant(m, n, p, A, B, k, split, rm, D2, &w);
        }
    bad += oz_dgemm_per_slice(m, n, p, A, B, k, D2, &w);
    oz_dot2_gemm(m, n, p, A, B, D2, D);
    oz_axpby(m, p, -1.75, D2, 0.3, D);
    oz_axpby(m, p, 2.0, D2, 0.0, D);
    if (m > 0 && n > 0 && p > 0) {
        /* phase entry points on exactly sized buffers */
        int32_t *eA = (int32_t *)malloc((size_t)m * sizeof(int32_t)), *eB = (int32_t *)malloc((size_t)p * sizeof(int32_t));
        int32_t *eK = (int32_t *)malloc((size_t)k * (size_t)(m > p ? m : p) * sizeof(int32_t));
        int8_t *SA = (int8_t *)malloc((size_t)k * (size_t)(m * n)), *SB = (int8_t *)malloc((size_t)k * (size_t)(n * p));
        int32_t *C = (int32_t *)malloc((size_t)(m * p) * sizeof(int32_t));
        for (int form = 0; form < 3; ++form) {
            if (form == 2) {
                oz_exponents_floor(m, n, A, 0, eA);
                oz_exponents_floor(n, p, B, 1, eB);
            } else {
                oz_row_exponents(m, n, A, eA);
                oz_col_exponents(n, p, B, eB);
            }
            oz_split_rows(m, n, A, eA, beta, k, form, SA);
            oz_split_cols(n, p, B, eB, beta, k, form, SB);
            for (int g = 2; g <= k + 1; ++g) {
                bad += oz_group_chunk(m, n, p, SA, SB, g, 1, 1, C);
                oz_accumulate(m, p, C, eA, eB, beta, g, g == 2, D);
            }
        }
        for (int form = 0; form < 2; ++form) {
            oz_split_per_slice(m, n, A, 0, beta, k, form, SA, eK);
            oz_split_per_slice(n, p, B, 1, beta, k, form, SB, eK);
        }
        free(eA); free(eB); free(eK); free(SA); free(SB); free(C);
    }
    free(A); free(B); free(D); free(D2);
    return bad != 0;
}

int main(void)
{
    int fails = 0;
    /* parameter functions over the whole admissible range of n */
    for (int64_t n = 1; n <= ((int64_t)1 << 29); n = n * 2 + (n & 1 ? 0 : 1)) {
        int beta = oz_beta(n);
        (void)oz_r(n, beta);
        (void)oz_r_wide(n, beta);
    }
    for (int k = 1; k <= 20; ++k)
        for (int64_t r = 1; r <= 64; r *= 2) (void)oz_count_addends(k, r);
    (void)oz_num_threads();
    fails += run_case(7, 33, 5, 6, 0.5, 1);
    fails += run_case(16, 64, 9, 20, 4.0, 1);
    fails += run_case(3, 300, 4, 8, 2.0, 0);
    fails += run_case(1, 1, 1, 1, 0.0, 0);
    fails += run_case(2, 0, 3, 4, 1.0, 0);
    fails += run_case(0, 5, 3, 4, 1.0, 0);
    if (fails) {
        printf("sanitize driver: %d case(s) reported INT32 overflow\n", fails);
        return 1;
    }
    printf("sanitize driver ok\n");
    return 0;
}
