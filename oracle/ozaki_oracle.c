/*
 * CPU oracle for FP64 GEMM emulation on an INT8 matrix unit (Ozaki scheme,
 * round-to-nearest slices with one power-of-two scale per row / column,
 * group-wise error-free INT32 accumulation, shifted FP64 accumulation).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, scalar checker that
 * the GPU library is compared against.  It shares no code, header, table or
 * helper with the GPU path, and the product never calls it.
 *
 * Notation follows the paper: A is m x n, B is n x p (n is the inner
 * dimension), D is m x p, k slices, beta bits per slice, r products per
 * error-free INT32 group.  All matrices are dense row-major with no padding.
 *
 * Every function cites the passage it follows (section / equation /
 * algorithm).  Pins for every function live in tests/test_oracle_*.py.
 * Parity unpinned: nothing in this file (absolute accuracy levels of the
 * paper's figures cannot be reproduced because the plots are not available,
 * but no function here depends on them).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* Parameters                                                          */
/* ------------------------------------------------------------------ */

/* beta = min(7, floor((31 - log2 n)/2))            [Section 2, the formula for beta]
 * Integer form: floor((31 - log2 n)/2) >= b  <=>  n <= 2^(31-2b).
 * Returns 0 when even b = 1 does not fit (n > 2^29, outside the paper's
 * standing assumption beta >= 1). */
int oz_beta(int64_t n)
{
    int beta = 0;
    for (int b = 1; b <= 7; ++b) {
        if (n <= ((int64_t)1 << (31 - 2 * b))) beta = b;
    }
    return beta;
}

/* ceil(log2 n) for n >= 1: the smallest L with n <= 2^L. */
static int ceil_log2_i64(int64_t n)
{
    int L = 0;
    while (((int64_t)1 << L) < n) ++L;
    return L;
}

/* r = max(1, 2^(31 - 2 beta - ceil(log2 n)))        [Section 3.2, the definition of r] */
int64_t oz_r(int64_t n, int beta)
{
    int ex = 31 - 2 * beta - ceil_log2_i64(n);
    if (ex <= 0) return 1;
    return (int64_t)1 << ex;
}

/* Number of FP64 addends produced by the chunked accumulation, counted by
 * walking the loops of Algorithm 6 (used to pin the walk against the closed
 * form w of Section 5.2). */
int64_t oz_count_addends(int k, int64_t r)
{
    int64_t w = 0;
    for (int g = 2; g <= k + 1; ++g) {
        int64_t q = 0;
        for (int s = 1; s <= g - 1; ++s) {
            ++q;
            if (q == r || s == g - 1) { ++w; q = 0; }
        }
    }
    return w;
}

/* ------------------------------------------------------------------ */
/* Step (i)/(ii): power-of-two scale exponents                         */
/* ------------------------------------------------------------------ */

/* e = ceil(log2 x) for finite x > 0 without calling log2 (Section 2 warns
 * that log2 may return a wrong integer): write x = f * 2^t with
 * f in [0.5, 1); then x <= 2^t always, and x <= 2^(t-1) only if f = 0.5. */
static int ceil_log2_double(double x)
{
    int t;
    double f = frexp(x, &t);
    return (f == 0.5) ? t - 1 : t;
}

/* eA[i] = ceil(log2 max_j |a_ij|)         [Algorithm 8, the exponent part of its scale mu'']
 * An all-zero row gets exponent 0 (every slice of it is zero). */
void oz_row_exponents(int64_t m, int64_t n, const double *A, int32_t *eA)
{
    for (int64_t i = 0; i < m; ++i) {
        double mx = 0.0;
        for (int64_t j = 0; j < n; ++j) {
            double v = fabs(A[i * n + j]);
            if (v > mx) mx = v;
        }
        eA[i] = (mx > 0.0) ? ceil_log2_double(mx) : 0;
    }
}

/* Scale exponents of the bit-mask split of the earlier ozIMMU method: floor instead of ceil,
 * mu''_i = 2^floor(log2 max_j |a_ij|)                                  [Algorithm 3, its scale mu'']
 * (x = f * 2^t with f in [0.5, 1) has floor(log2 x) = t - 1).  cols != 0: per column of an n x p matrix. */
void oz_exponents_floor(int64_t rows, int64_t cols_, const double *X, int by_col, int32_t *e)
{
    int64_t nvec = by_col ? cols_ : rows, len = by_col ? rows : cols_;
    for (int64_t v = 0; v < nvec; ++v) {
        double mx = 0.0;
        for (int64_t l = 0; l < len; ++l) {
            double x = fabs(by_col ? X[l * cols_ + v] : X[v * cols_ + l]);
            if (x > mx) mx = x;
        }
        int t = 0;
        if (mx > 0.0) { (void)frexp(mx, &t); t -= 1; }
        e[v] = t;
    }
}

/* eB[j] = ceil(log2 max_i |b_ij|): B is split as the transpose of the split
 * of B^T (Section 2, the remark after the expansions of A and B), i.e. one scale per column. */
void oz_col_exponents(int64_t n, int64_t p, const double *B, int32_t *eB)
{
    for (int64_t j = 0; j < p; ++j) {
        double mx = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            double v = fabs(B[i * p + j]);
            if (v > mx) mx = v;
        }
        eB[j] = (mx > 0.0) ? ceil_log2_double(mx) : 0;
    }
}

/* ------------------------------------------------------------------ */
/* Step (i)/(ii): slice extraction                                     */
/* ------------------------------------------------------------------ */

/* Round-to-nearest-even slices of ONE number a with scale exponent e
 * (|a| <= 2^e), in exact integer arithmetic.       [Algorithm 8, the loop over the slices]
 *
 * Slice s lives on the grid 2^(e+1-s*beta) (= mu'' * 2^(-beta(s-1)) with
 * mu'' = 2^e * 2^(1-beta)); q_s is the integer nearest to remainder/grid,
 * ties to even, and the remainder is reduced by q_s * grid.  The remainder is
 * held as N * 2^X with N a signed 64-bit integer, so nothing is rounded
 * except where the algorithm rounds. */
static void split_one_int(double a, int e, int beta, int k, int8_t *q, int64_t stride)
{
    int t;
    double f = frexp(a, &t);                  /* a = f * 2^t, |f| in [0.5,1) or 0 */
    int64_t N = (int64_t)ldexp(f, 53);        /* exact: 53-bit signed integer */
    int X = t - 53;                           /* a = N * 2^X */
    for (int s = 1; s <= k; ++s) {
        int gexp = e + 1 - s * beta;          /* grid = 2^gexp */
        int d = gexp - X;                     /* remainder / grid = N / 2^d */
        int64_t qs;
        if (N == 0) {
            qs = 0;
        } else if (d <= 0) {
            qs = N * ((int64_t)1 << (-d));    /* already an integer multiple of the grid */
            N = 0;
        } else if (d >= 62) {
            qs = 0;                           /* |N| < 2^54 << half a grid step */
        } else {
            int64_t one = (int64_t)1 << d;
            int64_t fl = N >> d;              /* floor(N / 2^d) (arithmetic shift) */
            int64_t rem = N - fl * one;       /* 0 <= rem < 2^d */
            int64_t half = one >> 1;
            if (rem > half || (rem == half && (fl & 1))) fl += 1;
            qs = fl;
            N -= qs * one;
        }
        q[(int64_t)(s - 1) * stride] = (int8_t)qs;
    }
}

/* The same slices by the floating-point recipe printed in Algorithm 8:
 * mu = 2^e * 2^(1-beta); sigma = 0.75 * 2^(53-beta(s-1)) * mu;
 * A_s = (a + sigma) - sigma in FP64 round-to-nearest-even;
 * q_s = A_s / (mu * 2^(-beta(s-1))); a <- a - A_s.
 * (The index garbles of the printed listing are read as: loop index i over
 * rows; the INT8 value is A_s divided by the slice grid.)  volatile keeps the
 * compiler from simplifying (a + sigma) - sigma. */
static void split_one_sigma(double a, int e, int beta, int k, int8_t *q, int64_t stride)
{
    double mu = ldexp(1.0, e + 1 - beta);
    for (int s = 1; s <= k; ++s) {
        double grid = ldexp(mu, -beta * (s - 1));
        volatile double sigma = 0.75 * ldexp(grid, 53);
        volatile double t = a + sigma;
        double As = t - sigma;
        q[(int64_t)(s - 1) * stride] = (int8_t)(As / grid);
        a = a - As;
    }
}

/* Bit-mask slices of ONE number a with scale exponent e = floor(log2 max) (|a| < 2^(e+1)):
 * slice s holds the s-th group of beta bits of |a| below 2^(e+1), with the sign of a, i.e. the
 * remainder divided by the grid 2^(e+1-s*beta) and truncated toward zero; |q_s| <= 2^beta - 1.
 *                                           [the digit extraction of Algorithm 3; the expansion of A in Section 2]
 * The paper describes the earlier method only this far ("extract the s-th beta bits of the mantissa
 * via bit masking"); truncation toward zero of a sign-magnitude number is that operation. */
static void split_one_trunc(double a, int e, int beta, int k, int8_t *q, int64_t stride)
{
    int t;
    double f = frexp(a, &t);
    int64_t N = (int64_t)ldexp(f, 53);
    int X = t - 53;
    for (int s = 1; s <= k; ++s) {
        int gexp = e + 1 - s * beta;
        int d = gexp - X;
        int64_t qs;
        if (N == 0) {
            qs = 0;
        } else if (d <= 0) {
            qs = N * ((int64_t)1 << (-d));
            N = 0;
        } else if (d >= 62) {
            qs = 0;
        } else {
            int64_t mag = N < 0 ? -N : N;
            int64_t qm = mag >> d;                 /* floor of the magnitude */
            qs = N < 0 ? -qm : qm;
            N -= qs * ((int64_t)1 << d);
        }
        q[(int64_t)(s - 1) * stride] = (int8_t)qs;
    }
}

/* Slices of all of A: SA[s-1][i][j], s = 1..k, with row exponents eA given.
 * form = 0: integer form, form = 1: Algorithm 8's floating-point form, form = 2: bit-mask slices
 * of Algorithm 3 (eA must then hold floor exponents). */
void oz_split_rows(int64_t m, int64_t n, const double *A, const int32_t *eA,
                   int beta, int k, int form, int8_t *SA)
{
    int64_t stride = m * n;
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j) {
            if (form == 0)      split_one_int(A[i * n + j], eA[i], beta, k, SA + i * n + j, stride);
            else if (form == 1) split_one_sigma(A[i * n + j], eA[i], beta, k, SA + i * n + j, stride);
            else                split_one_trunc(A[i * n + j], eA[i], beta, k, SA + i * n + j, stride);
        }
}

/* Slices of all of B: SB[t-1][i][j] (same n x p shape as B), column scales. */
void oz_split_cols(int64_t n, int64_t p, const double *B, const int32_t *eB,
                   int beta, int k, int form, int8_t *SB)
{
    int64_t stride = n * p;
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < p; ++j) {
            if (form == 0)      split_one_int(B[i * p + j], eB[j], beta, k, SB + i * p + j, stride);
            else if (form == 1) split_one_sigma(B[i * p + j], eB[j], beta, k, SB + i * p + j, stride);
            else                split_one_trunc(B[i * p + j], eB[j], beta, k, SB + i * p + j, stride);
        }
}

/* Round-to-nearest slices with ONE SCALE PER SLICE (the first of the paper's two round-to-nearest
 * splits; it is the split of ozIMMU_RN).                              [Algorithm 5]
 * For s = 1..k: the scale exponent of slice s is taken from what is LEFT of the vector,
 *   e_s = ceil(log2 max |remainder|)   (0 when the remainder is all zero),
 *   mu'(s) = 2^(e_s + 1 - beta),  q_s = RNE(remainder / mu'(s)),  remainder <- remainder - q_s mu'(s).
 * |q_s| <= 2^(beta-1), and |remainder| <= mu'(s)/2 afterwards, so e_(s+1) <= e_s - beta.
 * X is rows x cols row-major; by_col == 0: one vector per row, by_col != 0: one vector per column
 * (B is split as the transpose of the split of B^T).  S[s-1] has the shape of X; E[s-1][v] = e_s of
 * vector v.  form 0: q by scaling with a power of two and rint (both exact but for the rounding that
 * the algorithm asks for); form 1: the (a + sigma) - sigma recipe as printed, sigma = 0.75 2^53 mu'(s). */
void oz_split_per_slice(int64_t rows, int64_t cols_, const double *X, int by_col, int beta, int k, int form,
                        int8_t *S, int32_t *E)
{
    int64_t nvec = by_col ? cols_ : rows, len = by_col ? rows : cols_;
    int64_t stride = rows * cols_;
    double *rem = (double *)malloc((size_t)(len > 0 ? len : 1) * sizeof(double));
    for (int64_t v = 0; v < nvec; ++v) {
        for (int64_t l = 0; l < len; ++l) rem[l] = by_col ? X[l * cols_ + v] : X[v * cols_ + l];
        for (int s = 1; s <= k; ++s) {
            double mx = 0.0;
            for (int64_t l = 0; l < len; ++l) {
                double a = fabs(rem[l]);
                if (a > mx) mx = a;
            }
            int e = (mx > 0.0) ? ceil_log2_double(mx) : 0;
            E[(int64_t)(s - 1) * nvec + v] = e;
            double mu = ldexp(1.0, e + 1 - beta);
            for (int64_t l = 0; l < len; ++l) {
                double As;
                if (form == 0) {
                    As = ldexp(rint(ldexp(rem[l], beta - 1 - e)), e + 1 - beta);
                } else {
                    volatile double sigma = 0.75 * ldexp(mu, 53);
                    volatile double t = rem[l] + sigma;
                    As = t - sigma;
                }
                int64_t at = by_col ? l * cols_ + v : v * cols_ + l;
                S[(int64_t)(s - 1) * stride + at] = (int8_t)(As / mu);
                rem[l] -= As;
            }
        }
    }
    free(rem);
}

/* ------------------------------------------------------------------ */
/* Step (iii): integer products                                        */
/* ------------------------------------------------------------------ */

/* C'' = sum_{s=s0..s1} A''_s B''_{g-s} for one chunk of one group
 *                                   [inner loop of Algorithm 6; the grouped sum of Section 3.2]
 * Dot products are taken in int64 and every chunk sum is checked to fit
 * INT32 (the overflow bound of Section 5.2).  s0 == s1 gives one slice pair
 * A''_s B''_t of Algorithm 4.  Returns the number of results that did NOT fit
 * (0 expected); results are stored truncated to int32 either way. */
int64_t oz_group_chunk(int64_t m, int64_t n, int64_t p,
                       const int8_t *SA, const int8_t *SB,
                       int g, int s0, int s1, int32_t *C)
{
    int64_t bad = 0;
#pragma omp parallel for schedule(static) reduction(+ : bad)
    for (int64_t i = 0; i < m; ++i) {
        int64_t *acc = (int64_t *)calloc((size_t)p, sizeof(int64_t));
        for (int s = s0; s <= s1; ++s) {
            const int8_t *As = SA + (int64_t)(s - 1) * m * n;
            const int8_t *Bt = SB + (int64_t)(g - s - 1) * n * p;
            for (int64_t l = 0; l < n; ++l) {
                int64_t a = As[i * n + l];
                const int8_t *brow = Bt + l * p;
                for (int64_t j = 0; j < p; ++j) acc[j] += a * (int64_t)brow[j];
            }
        }
        for (int64_t j = 0; j < p; ++j) {
            if (acc[j] > INT32_MAX || acc[j] < INT32_MIN) ++bad;
            C[i * p + j] = (int32_t)acc[j];
        }
        free(acc);
    }
    return bad;
}

/* ------------------------------------------------------------------ */
/* Step (iv): shifted FP64 accumulation                                */
/* ------------------------------------------------------------------ */

/* D <- D + 2^(-beta g + 2) diag(2^eA) FP64(C'') diag(2^eB)
 *                                                     [Algorithm 6, the accumulation step]
 * (mu'', nu'' of the expansions of A and B in Section 2 are 2^eA, 2^eB.)  The conversion
 * and the power-of-two scaling are exact; the addition is the only rounding.
 * first != 0 means D is the zero matrix (the initialisation D = O of Algorithm 6). */
void oz_accumulate(int64_t m, int64_t p, const int32_t *C,
                   const int32_t *eA, const int32_t *eB,
                   int beta, int g, int first, double *D)
{
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < p; ++j) {
            double term = ldexp((double)C[i * p + j], eA[i] + eB[j] + 2 - beta * g);
            double d = first ? 0.0 : D[i * p + j];
            D[i * p + j] = d + term;
        }
}

/* ------------------------------------------------------------------ */
/* Whole path                                                          */
/* ------------------------------------------------------------------ */

/* Largest power of two r_w with r_w * n * (2^(beta-1))^2 <= 2^31 - 1: the number of products of
 * round-to-nearest slices (|q| <= 2^(beta-1), tighter than the 2^beta - 1 behind the paper's r) that
 * can share an INT32 accumulator.  An option beyond the paper; never below the paper's r. */
int64_t oz_r_wide(int64_t n, int beta)
{
    int64_t r = 1;
    const int64_t lim = ((int64_t)1 << 31) - 1;
    while (2 * r * n * ((int64_t)1 << (2 * beta - 2)) <= lim) r *= 2;
    return r;
}

/* D = A B emulated with k slices, in the variants the paper compares (Section 4):
 *   split_mode 0: round-to-nearest slices, one scale per row/column     [Algorithm 8]
 *   split_mode 1: bit-mask slices                                        [Algorithm 3]
 *   r_mode 0: chunks of r products (Section 3.2)                        [Algorithm 6]
 *   r_mode 1: one FP64 addition per slice pair                           [Algorithm 4]
 *   r_mode 2: chunks of oz_r_wide products (split_mode 0 only; beyond the paper)
 * (0,0) = ozIMMU_H, (1,0) = ozIMMU_EF, (1,1) = ozIMMU.
 * A is m x n, B is n x p, both dense row-major; D (m x p) is overwritten.
 * Returns 0, or -1 for arguments outside the method's domain, or the number
 * of INT32 overflows (never expected).  *n_addends (optional) receives the
 * number of FP64 additions per element of D. */
int64_t oz_dgemm_variant(int64_t m, int64_t n, int64_t p, const double *A, const double *B,
                         int k, int split_mode, int r_mode, double *D, int64_t *n_addends)
{
    if (m < 0 || n < 0 || p < 0 || k < 1) return -1;
    if (split_mode < 0 || split_mode > 1 || r_mode < 0 || r_mode > 2 || (r_mode == 2 && split_mode != 0)) return -1;
    for (int64_t x = 0; x < m * p; ++x) D[x] = 0.0;
    if (n_addends) *n_addends = 0;
    if (m == 0 || p == 0 || n == 0) return 0;
    int beta = oz_beta(n);
    if (beta < 1) return -1;
    int64_t r = r_mode == 0 ? oz_r(n, beta) : (r_mode == 1 ? 1 : oz_r_wide(n, beta));

    int32_t *eA = (int32_t *)malloc((size_t)m * sizeof(int32_t));
    int32_t *eB = (int32_t *)malloc((size_t)p * sizeof(int32_t));
    int8_t *SA = (int8_t *)malloc((size_t)k * m * n);
    int8_t *SB = (int8_t *)malloc((size_t)k * n * p);
    int32_t *C = (int32_t *)malloc((size_t)m * p * sizeof(int32_t));

    if (split_mode == 0) {
        oz_row_exponents(m, n, A, eA);
        oz_col_exponents(n, p, B, eB);
        oz_split_rows(m, n, A, eA, beta, k, 0, SA);
        oz_split_cols(n, p, B, eB, beta, k, 0, SB);
    } else {
        oz_exponents_floor(m, n, A, 0, eA);
        oz_exponents_floor(n, p, B, 1, eB);
        oz_split_rows(m, n, A, eA, beta, k, 2, SA);
        oz_split_cols(n, p, B, eB, beta, k, 2, SB);
    }

    int64_t bad = 0, w = 0;
    int first = 1;
    for (int g = 2; g <= k + 1; ++g) {
        int64_t q = 0;      /* products gathered in the open chunk */
        int s_open = 1;     /* first s of the open chunk */
        for (int s = 1; s <= g - 1; ++s) {
            ++q;
            if (q == r || s == g - 1) {
                bad += oz_group_chunk(m, n, p, SA, SB, g, s_open, s, C);
                oz_accumulate(m, p, C, eA, eB, beta, g, first, D);
                first = 0;
                ++w;
                q = 0;
                s_open = s + 1;
            }
        }
    }
    if (n_addends) *n_addends = w;
    free(eA); free(eB); free(SA); free(SB); free(C);
    return bad;
}

/* D = A B by ozIMMU_RN: slices with one scale per slice (Algorithm 5), and one FP64 addition per
 * slice pair with s + t <= k + 1 in the order g = s + t ascending, s ascending:
 *   D <- D + diag(mu'(s)) FP64(A'_s B'_t) diag(nu'(t)),  mu'(s)_i nu'(t)_j = 2^(eA_s[i] + eB_t[j] + 2 - 2 beta)
 *                                      [Algorithm 5; accumulation in the form of Algorithms 2 and 4]
 * Same return values as oz_dgemm_variant. */
int64_t oz_dgemm_per_slice(int64_t m, int64_t n, int64_t p, const double *A, const double *B,
                           int k, double *D, int64_t *n_addends)
{
    if (m < 0 || n < 0 || p < 0 || k < 1) return -1;
    for (int64_t x = 0; x < m * p; ++x) D[x] = 0.0;
    if (n_addends) *n_addends = 0;
    if (m == 0 || p == 0 || n == 0) return 0;
    int beta = oz_beta(n);
    if (beta < 1) return -1;
    int32_t *eA = (int32_t *)malloc((size_t)k * m * sizeof(int32_t));
    int32_t *eB = (int32_t *)malloc((size_t)k * p * sizeof(int32_t));
    int8_t *SA = (int8_t *)malloc((size_t)k * m * n);
    int8_t *SB = (int8_t *)malloc((size_t)k * n * p);
    int32_t *C = (int32_t *)malloc((size_t)m * p * sizeof(int32_t));
    oz_split_per_slice(m, n, A, 0, beta, k, 0, SA, eA);
    oz_split_per_slice(n, p, B, 1, beta, k, 0, SB, eB);
    int64_t bad = 0, w = 0;
    for (int g = 2; g <= k + 1; ++g)
        for (int s = 1; s <= g - 1; ++s) {
            int t = g - s;
            bad += oz_group_chunk(m, n, p, SA, SB, g, s, s, C);
            /* oz_accumulate with g = 2 applies 2^(e + f + 2 - 2 beta) */
            oz_accumulate(m, p, C, eA + (int64_t)(s - 1) * m, eB + (int64_t)(t - 1) * p, beta, 2, w == 0, D);
            ++w;
        }
    if (n_addends) *n_addends = w;
    free(eA); free(eB); free(SA); free(SB); free(C);
    return bad;
}

/* D = A B emulated with k slices.            [Algorithm 8 + Algorithm 6] */
int64_t oz_dgemm(int64_t m, int64_t n, int64_t p, const double *A, const double *B,
                 int k, double *D, int64_t *n_addends)
{
    return oz_dgemm_variant(m, n, p, A, B, k, 0, 0, D, n_addends);
}

/* ------------------------------------------------------------------ */
/* Accuracy reference: compensated dot product                         */
/* ------------------------------------------------------------------ */

/* R = A B with every dot product evaluated by the Dot2 algorithm of Ogita,
 * Rump and Oishi: TwoProduct (with a fused multiply-add) and TwoSum error-free
 * transformations, the error terms summed in a second double.  The result is
 * as accurate as if computed in twice the working precision and is returned
 * UNEVALUATED as hi + lo so that errors below one ulp can still be measured.
 * Not part of the method; it is the yardstick the paper's accuracy plots use
 * an accurate product for (Section 4.1). */
void oz_dot2_gemm(int64_t m, int64_t n, int64_t p, const double *A, const double *B,
                  double *Rhi, double *Rlo)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        double *ph = (double *)calloc((size_t)p, sizeof(double));
        double *sl = (double *)calloc((size_t)p, sizeof(double));
        for (int64_t l = 0; l < n; ++l) {
            double a = A[i * n + l];
            const double *brow = B + l * p;
            for (int64_t j = 0; j < p; ++j) {
                double h = a * brow[j];
                double rr = fma(a, brow[j], -h);          /* TwoProduct */
                double x = ph[j] + h;                      /* TwoSum(ph, h) */
                double z = x - ph[j];
                double y = (ph[j] - (x - z)) + (h - z);
                ph[j] = x;
                sl[j] += (y + rr);
            }
        }
        for (int64_t j = 0; j < p; ++j) {
            /* renormalise so that |lo| <= ulp(hi)/2 */
            double x = ph[j] + sl[j];
            double z = x - ph[j];
            double y = (ph[j] - (x - z)) + (sl[j] - z);
            Rhi[i * p + j] = x;
            Rlo[i * p + j] = y;
        }
        free(ph); free(sl);
    }
}

int oz_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Step (v): C <- alpha D + beta C                                     */
/* ------------------------------------------------------------------ */

/* The fifth step of the scheme when a GEMM routine is emulated (Section 1):
 * C <- alpha * D + beta * C with D the emulated product.  The paper gives no
 * rounding order; the reading taken is the plain one, three rounded FP64
 * operations per element, t1 = fl(alpha d), t2 = fl(beta c), c = fl(t1 + t2),
 * no fused multiply-add, and the BLAS convention that beta == 0 means C is not
 * read (c = fl(alpha d), so that NaN or Inf in the old C does not propagate). */
void oz_axpby(int64_t m, int64_t p, double alpha, const double *D, double beta, double *C)
{
    for (int64_t x = 0; x < m * p; ++x) {
        volatile double t1 = alpha * D[x];
        if (beta == 0.0) {
            C[x] = t1;
        } else {
            volatile double t2 = beta * C[x];
            C[x] = t1 + t2;
        }
    }
}
