/*
 * CPU oracle for the f16 GEMM hot path.  TEST INFRASTRUCTURE ONLY: nothing in
 * the product path may call, link or import this file; it shares no code with
 * the HIP kernels.
 *
 * What it computes is the plain definition of the paper's problem statement
 * (Evaluation section: C = A B + C, all three matrices row-major; Listing
 * "Naive affine matmul": every product of two f16 inputs is widened and added
 * to C[i][j], for k = 0 .. K-1):
 *
 *     C_ref[i][j] = C0[i][j] + sum_{k=0}^{K-1} A[i][k] * B[k][j]
 *
 * evaluated in IEEE binary64, one term at a time in increasing k, together
 * with the magnitude sum
 *
 *     S[i][j]     = sum_{k=0}^{K-1} |A[i][k]| * |B[k][j]|
 *
 * that the parity tolerances are scaled by.  An f16 value converts to binary64
 * exactly and a product of two f16 values has at most 22 significant bits, so
 * every product is exact in binary64; the only rounding is in the running sum
 * (relative error at most K * 2^-53 of S).  The same function serves both
 * modes of the paper (Mixed Precision Performance: C in f32; Half Precision
 * Performance: C in f16): only the storage type of C0 differs, and the result
 * stays in binary64 so that a test can compare against it or round it once.
 *
 * There is no blocking, fusion or reordering: three nested loops (i, k, j —
 * for each output element the terms still arrive in increasing k) and an
 * OpenMP "parallel for" over the rows i, which are independent.
 *
 * Pins (tests/test_oracle_*.py, CPU only): f16 decoder against numpy for all
 * 65536 bit patterns; f64->f32/f16 encoders against numpy; identity,
 * permutation, all-ones, rank-1 and index-product closed forms; exact rational
 * arithmetic on tiny shapes; numpy's f64 matmul on integer-valued inputs
 * (exact); scaling, transpose and S >= |C_ref - C0| invariants.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* IEEE binary16 bit pattern -> binary64 value (exact).  Sign 1 bit, exponent 5
 * bits (bias 15), fraction 10 bits; exponent 0 is zero/subnormal
 * (frac * 2^-24), exponent 31 is inf/NaN. */
double oracle_f16_bits_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (e == 0) {
        v = ldexp((double)frac, -24);
    } else if (e == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + frac), e - 25);
    }
    return sign ? -v : v;
}

/* binary32 bit pattern -> binary64 (exact). Written out rather than cast so
 * that the decoder is checkable on its own. */
double oracle_f32_bits_to_f64(uint32_t w)
{
    int sign = (w >> 31) & 1;
    int e = (w >> 23) & 0xff;
    uint32_t frac = w & 0x7fffffu;
    double v;
    if (e == 0) {
        v = ldexp((double)frac, -149);
    } else if (e == 255) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(0x800000u + frac), e - 150);
    }
    return sign ? -v : v;
}

/* Round a binary64 value to the nearest value with `pbits` significand bits
 * (implicit bit included), minimum normal exponent `emin` and largest finite
 * exponent `emax` (value = m * 2^e, 1 <= m < 2), ties to even; overflow goes to
 * infinity, tiny values go through the subnormal grid 2^(emin - pbits + 1).
 * Returns the rounded value as a double (exactly representable). */
static double round_to_format(double x, int pbits, int emin, int emax)
{
    if (isnan(x) || isinf(x) || x == 0.0) return x;
    int ex;
    double m = frexp(fabs(x), &ex); /* |x| = m * 2^ex, 0.5 <= m < 1 */
    int e = ex - 1;                 /* |x| = (2m) * 2^e, 1 <= 2m < 2 */
    if (e < emin) e = emin;         /* subnormal range: fixed grid */
    /* grid spacing at this exponent */
    int q = e - (pbits - 1);
    double scaled = ldexp(fabs(x), -q); /* exact: power-of-two scaling */
    double r = nearbyint(scaled);       /* default rounding mode: ties to even */
    (void)m;
    double y = ldexp(r, q);
    /* overflow: anything that rounds to 2^(emax+1) or above is infinite */
    if (y >= ldexp(1.0, emax + 1)) y = INFINITY;
    return x < 0 ? -y : y;
}

static uint16_t f64_exact_to_f16_bits(double y)
{
    uint16_t sign = signbit(y) ? 0x8000u : 0;
    double a = fabs(y);
    if (isnan(y)) return 0x7e00u;
    if (isinf(a)) return sign | 0x7c00u;
    if (a == 0.0) return sign;
    if (a < ldexp(1.0, -14)) { /* subnormal */
        return sign | (uint16_t)ldexp(a, 24);
    }
    int ex;
    double m = frexp(a, &ex); /* a = m 2^ex */
    int e = ex - 1;
    uint32_t frac = (uint32_t)ldexp(m, 11) - 1024u; /* (2m) * 2^10 - 2^10 */
    return sign | (uint16_t)((e + 15) << 10) | (uint16_t)frac;
}

/* binary64 -> binary16 bits, single rounding, ties to even. */
uint16_t oracle_f64_to_f16_bits(double x)
{
    return f64_exact_to_f16_bits(round_to_format(x, 11, -14, 15));
}

/* binary64 -> binary32 bits, single rounding, ties to even. */
uint32_t oracle_f64_to_f32_bits(double x)
{
    double y = round_to_format(x, 24, -126, 127);
    uint32_t sign = signbit(y) ? 0x80000000u : 0;
    double a = fabs(y);
    if (isnan(y)) return 0x7fc00000u;
    if (isinf(a)) return sign | 0x7f800000u;
    if (a == 0.0) return sign;
    if (a < ldexp(1.0, -126)) return sign | (uint32_t)ldexp(a, 149);
    int ex;
    double m = frexp(a, &ex);
    int e = ex - 1;
    uint32_t frac = (uint32_t)ldexp(m, 24) - 0x800000u;
    return sign | ((uint32_t)(e + 127) << 23) | frac;
}

/* array forms, for the Python side */
void oracle_f16_bits_to_f64_array(const uint16_t* h, double* out, int64_t n)
{
    for (int64_t i = 0; i < n; i++) out[i] = oracle_f16_bits_to_f64(h[i]);
}
void oracle_f64_to_f16_bits_array(const double* x, uint16_t* out, int64_t n)
{
    for (int64_t i = 0; i < n; i++) out[i] = oracle_f64_to_f16_bits(x[i]);
}
void oracle_f64_to_f32_bits_array(const double* x, uint32_t* out, int64_t n)
{
    for (int64_t i = 0; i < n; i++) out[i] = oracle_f64_to_f32_bits(x[i]);
}

/*
 * The oracle proper, on a chosen set of output rows.
 *
 *   M, N, K     problem size (A is M x K, B is K x N, C is M x N)
 *   A, lda      host pointer to f16 bit patterns, row-major, row pitch lda >= K
 *   B, ldb      likewise, row pitch ldb >= N
 *   C0, ldc     host pointer to the initial C: f32 bit patterns (c_is_f16 = 0)
 *               or f16 bit patterns (c_is_f16 = 1), row pitch ldc >= N
 *   rows, nrows the output rows wanted (each in [0, M)); rows == NULL means
 *               all M rows in order (then nrows must equal M)
 *   Cref, S     host outputs, nrows x N dense binary64; row r of the output is
 *               row rows[r] of the full result
 *
 * Returns 0, or a negative code: -1 bad size, -2 bad pitch, -3 null pointer,
 * -4 row index out of range, -5 out of memory.
 */
int oracle_gemm_f16_rows(int64_t M, int64_t N, int64_t K,
                         const uint16_t* A, int64_t lda,
                         const uint16_t* B, int64_t ldb,
                         const void* C0, int64_t ldc, int c_is_f16,
                         const int64_t* rows, int64_t nrows,
                         double* Cref, double* S)
{
    if (M < 0 || N < 0 || K < 0 || nrows < 0) return -1;
    if (lda < K || ldb < N || ldc < N) return -2;
    if (rows == NULL && nrows != M) return -1;
    if (nrows == 0 || N == 0) return 0;
    if (!C0 || !Cref || !S) return -3;
    if (K > 0 && (!A || !B)) return -3;
    if (rows)
        for (int64_t r = 0; r < nrows; r++)
            if (rows[r] < 0 || rows[r] >= M) return -4;

    /* B decoded once to binary64 (exact), dense K x N */
    double* Bd = NULL;
    if (K > 0) {
        Bd = (double*)malloc(sizeof(double) * (size_t)K * (size_t)N);
        if (!Bd) return -5;
#pragma omp parallel for schedule(static)
        for (int64_t k = 0; k < K; k++)
            for (int64_t j = 0; j < N; j++)
                Bd[k * N + j] = oracle_f16_bits_to_f64(B[k * ldb + j]);
    }

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < nrows; r++) {
        int64_t i = rows ? rows[r] : r;
        double* c = Cref + r * N;
        double* s = S + r * N;
        for (int64_t j = 0; j < N; j++) {
            if (c_is_f16)
                c[j] = oracle_f16_bits_to_f64(((const uint16_t*)C0)[i * ldc + j]);
            else
                c[j] = oracle_f32_bits_to_f64(((const uint32_t*)C0)[i * ldc + j]);
            s[j] = 0.0;
        }
        for (int64_t k = 0; k < K; k++) {
            double a = oracle_f16_bits_to_f64(A[i * lda + k]);
            double aa = fabs(a);
            const double* b = Bd + k * N;
            for (int64_t j = 0; j < N; j++) {
                c[j] += a * b[j];
                s[j] += aa * fabs(b[j]);
            }
        }
    }
    free(Bd);
    return 0;
}

/* All rows. */
int oracle_gemm_f16(int64_t M, int64_t N, int64_t K,
                    const uint16_t* A, int64_t lda,
                    const uint16_t* B, int64_t ldb,
                    const void* C0, int64_t ldc, int c_is_f16,
                    double* Cref, double* S)
{
    return oracle_gemm_f16_rows(M, N, K, A, lda, B, ldb, C0, ldc, c_is_f16,
                                NULL, M, Cref, S);
}

/* number of threads the row loop runs on */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
