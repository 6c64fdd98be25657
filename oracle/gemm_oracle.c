/*
 * CPU oracle for dense matrix multiplication  C = A * B.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the reference the GPU library is
 * checked against.  It shares no code with the GPU path and nothing in the
 * product may call it; only the tests, the smoke check and the benchmark's
 * CPU-baseline leg do.
 *
 * What it computes is the paper's MatMul specification (Section 3.1,
 * "Specifications"): A is M x K, B is K x N, C is M x N, and
 *
 *        C(i,j) = sum_{k = 0 .. K-1}  A(i,k) * B(k,j).
 *
 * C is overwritten: the paper's epilogue (Section 3.2, "Epilog") zero-fills
 * the accumulator and then stores it, so there is no alpha, beta or
 * accumulate-into-C.  K == 0 therefore yields C == 0.
 *
 * The GPU path reaches this sum exactly up to rounding order, so the oracle
 * is the definition written out: one scalar float64 accumulator per output
 * element, products added in ascending k.  Operands are widened to float64
 * first; a binary16 x binary16, bfloat16 x bfloat16 or binary32 x binary32
 * product is exact in float64, so the only error is the accumulation rounding (<= K * 2^-53
 * relative to sum |a*b|).  The result is returned as float64.
 *
 * Storage: element (r,c) of a row-major matrix with leading dimension ld sits
 * at index r*ld + c, of a column-major matrix at r + c*ld.  Each operand
 * carries its own layout flag (0 = row-major, 1 = column-major), as in the
 * paper's spec where every matrix records its storage layout.
 *
 * All pointers are HOST pointers.  Return value: 0 on success, -1 on an
 * invalid argument (negative size, bad layout flag, leading dimension below
 * the packed minimum, null pointer for a non-empty matrix).
 *
 * Parity pins (tests marked "not gpu"): brute force in Python integers on
 * tiny shapes, identity and permutation operands, the transpose invariant,
 * small-integer inputs against an int64 loop, closed forms, and a float64
 * numpy.matmul cross-check; for the binary16 rounding: the round trip of all
 * 65536 patterns, hand constants, exact midpoints (ties to even), the overflow
 * and subnormal thresholds, and numpy's float64 -> float16 conversion; for the
 * bfloat16 widening: all 65536 patterns against the binary32 number with the same upper
 * half, and hand constants.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_ROW_MAJOR = 0, ORACLE_COL_MAJOR = 1 };

/* index of element (r,c) */
static size_t at(int layout, int64_t ld, int64_t r, int64_t c)
{
    return layout == ORACLE_ROW_MAJOR ? (size_t)r * (size_t)ld + (size_t)c
                                      : (size_t)r + (size_t)c * (size_t)ld;
}

static int bad_matrix(const void *p, int layout, int64_t ld, int64_t rows, int64_t cols)
{
    if (layout != ORACLE_ROW_MAJOR && layout != ORACLE_COL_MAJOR) return 1;
    int64_t min_ld = layout == ORACLE_ROW_MAJOR ? cols : rows;
    if (ld < min_ld) return 1;
    if (rows > 0 && cols > 0 && p == NULL) return 1;
    return 0;
}

/* IEEE 754 binary16 bit pattern -> double, exact (every binary16 is a double). */
double oracle_half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        /* zero or subnormal: frac * 2^-24 */
        v = (double)frac * (1.0 / 16777216.0);
    } else if (expo == 31) {
        if (frac == 0) {
            v = 1.0 / 0.0;
        } else {
            v = 0.0 / 0.0;
        }
    } else {
        /* (1 + frac/1024) * 2^(expo-15) */
        v = 1.0 + (double)frac / 1024.0;
        int e = expo - 15;
        while (e > 0) { v *= 2.0; --e; }
        while (e < 0) { v *= 0.5; ++e; }
    }
    return sign ? -v : v;
}

/*
 * bfloat16 bit pattern -> double, exact.  The format is the upper half of IEEE binary32:
 * 1 sign bit, 8 exponent bits (bias 127), 7 fraction bits; normal numbers are
 * (1 + f/128) * 2^(e-127) with 1 <= e <= 254, subnormals f * 2^-133, e == 255 is
 * infinity (f == 0) or NaN.  Used by the bfloat16-operand sibling of the half-precision
 * product (same specification, Section 3.1; the tensor-core instruction of Section 4.2
 * with the other 16-bit operand format of the target).
 */
double oracle_bfloat16_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 7) & 0xff;
    int frac = h & 0x7f;
    double v;
    if (expo == 0) {
        v = (double)frac;
        for (int t = 0; t < 133; ++t) v *= 0.5;
    } else if (expo == 255) {
        if (frac == 0) {
            v = 1.0 / 0.0;
        } else {
            v = 0.0 / 0.0;
        }
    } else {
        v = 1.0 + (double)frac / 128.0;
        int e = expo - 127;
        while (e > 0) { v *= 2.0; --e; }
        while (e < 0) { v *= 0.5; ++e; }
    }
    return sign ? -v : v;
}

/*
 * Core: operands already widened to float64 in canonical form,
 *   a  : M x K, row-major, packed      (a[i*K + k]  = A(i,k))
 *   bt : N x K, row-major, packed      (bt[j*K + k] = B(k,j))
 * so the k loop walks both contiguously.  Ascending k, one accumulator.
 */
static void matmul_f64(int64_t M, int64_t N, int64_t K, const double *a, const double *bt,
                       double *C, int layoutC, int64_t ldc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += a[(size_t)i * K + k] * bt[(size_t)j * K + k];
            C[at(layoutC, ldc, i, j)] = acc;
        }
    }
}

int oracle_gemm_f32(int64_t M, int64_t N, int64_t K,
                    const float *A, int layoutA, int64_t lda,
                    const float *B, int layoutB, int64_t ldb,
                    double *C, int layoutC, int64_t ldc)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if (bad_matrix(A, layoutA, lda, M, K) || bad_matrix(B, layoutB, ldb, K, N) ||
        bad_matrix(C, layoutC, ldc, M, N))
        return -1;
    if (M == 0 || N == 0) return 0;
    double *a = (double *)malloc(sizeof(double) * (size_t)(M * K + 1));
    double *bt = (double *)malloc(sizeof(double) * (size_t)(N * K + 1));
    if (!a || !bt) { free(a); free(bt); return -2; }
    for (int64_t i = 0; i < M; ++i)
        for (int64_t k = 0; k < K; ++k) a[(size_t)i * K + k] = (double)A[at(layoutA, lda, i, k)];
    for (int64_t j = 0; j < N; ++j)
        for (int64_t k = 0; k < K; ++k) bt[(size_t)j * K + k] = (double)B[at(layoutB, ldb, k, j)];
    matmul_f64(M, N, K, a, bt, C, layoutC, ldc);
    free(a);
    free(bt);
    return 0;
}

int oracle_gemm_f16(int64_t M, int64_t N, int64_t K,
                    const uint16_t *A, int layoutA, int64_t lda,
                    const uint16_t *B, int layoutB, int64_t ldb,
                    double *C, int layoutC, int64_t ldc)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if (bad_matrix(A, layoutA, lda, M, K) || bad_matrix(B, layoutB, ldb, K, N) ||
        bad_matrix(C, layoutC, ldc, M, N))
        return -1;
    if (M == 0 || N == 0) return 0;
    double *a = (double *)malloc(sizeof(double) * (size_t)(M * K + 1));
    double *bt = (double *)malloc(sizeof(double) * (size_t)(N * K + 1));
    if (!a || !bt) { free(a); free(bt); return -2; }
    for (int64_t i = 0; i < M; ++i)
        for (int64_t k = 0; k < K; ++k)
            a[(size_t)i * K + k] = oracle_half_bits_to_double(A[at(layoutA, lda, i, k)]);
    for (int64_t j = 0; j < N; ++j)
        for (int64_t k = 0; k < K; ++k)
            bt[(size_t)j * K + k] = oracle_half_bits_to_double(B[at(layoutB, ldb, k, j)]);
    matmul_f64(M, N, K, a, bt, C, layoutC, ldc);
    free(a);
    free(bt);
    return 0;
}

int oracle_gemm_bf16(int64_t M, int64_t N, int64_t K,
                     const uint16_t *A, int layoutA, int64_t lda,
                     const uint16_t *B, int layoutB, int64_t ldb,
                     double *C, int layoutC, int64_t ldc)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if (bad_matrix(A, layoutA, lda, M, K) || bad_matrix(B, layoutB, ldb, K, N) ||
        bad_matrix(C, layoutC, ldc, M, N))
        return -1;
    if (M == 0 || N == 0) return 0;
    double *a = (double *)malloc(sizeof(double) * (size_t)(M * K + 1));
    double *bt = (double *)malloc(sizeof(double) * (size_t)(N * K + 1));
    if (!a || !bt) { free(a); free(bt); return -2; }
    for (int64_t i = 0; i < M; ++i)
        for (int64_t k = 0; k < K; ++k)
            a[(size_t)i * K + k] = oracle_bfloat16_bits_to_double(A[at(layoutA, lda, i, k)]);
    for (int64_t j = 0; j < N; ++j)
        for (int64_t k = 0; k < K; ++k)
            bt[(size_t)j * K + k] = oracle_bfloat16_bits_to_double(B[at(layoutB, ldb, k, j)]);
    matmul_f64(M, N, K, a, bt, C, layoutC, ldc);
    free(a);
    free(bt);
    return 0;
}

/*
 * Sampled form for sizes where the full product is too slow on a CPU: the same
 * definition evaluated only at the n listed positions (rows[t], cols[t]);
 * out[t] = C(rows[t], cols[t]).  Returns -1 if a position is out of range.
 */
int oracle_gemm_f32_at(int64_t M, int64_t N, int64_t K,
                       const float *A, int layoutA, int64_t lda,
                       const float *B, int layoutB, int64_t ldb,
                       int64_t n, const int64_t *rows, const int64_t *cols, double *out)
{
    if (M < 0 || N < 0 || K < 0 || n < 0) return -1;
    if (bad_matrix(A, layoutA, lda, M, K) || bad_matrix(B, layoutB, ldb, K, N)) return -1;
    for (int64_t t = 0; t < n; ++t)
        if (rows[t] < 0 || rows[t] >= M || cols[t] < 0 || cols[t] >= N) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k)
            acc += (double)A[at(layoutA, lda, rows[t], k)] * (double)B[at(layoutB, ldb, k, cols[t])];
        out[t] = acc;
    }
    return 0;
}

int oracle_gemm_f16_at(int64_t M, int64_t N, int64_t K,
                       const uint16_t *A, int layoutA, int64_t lda,
                       const uint16_t *B, int layoutB, int64_t ldb,
                       int64_t n, const int64_t *rows, const int64_t *cols, double *out)
{
    if (M < 0 || N < 0 || K < 0 || n < 0) return -1;
    if (bad_matrix(A, layoutA, lda, M, K) || bad_matrix(B, layoutB, ldb, K, N)) return -1;
    for (int64_t t = 0; t < n; ++t)
        if (rows[t] < 0 || rows[t] >= M || cols[t] < 0 || cols[t] >= N) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k)
            acc += oracle_half_bits_to_double(A[at(layoutA, lda, rows[t], k)]) *
                   oracle_half_bits_to_double(B[at(layoutB, ldb, k, cols[t])]);
        out[t] = acc;
    }
    return 0;
}

int oracle_gemm_bf16_at(int64_t M, int64_t N, int64_t K,
                        const uint16_t *A, int layoutA, int64_t lda,
                        const uint16_t *B, int layoutB, int64_t ldb,
                        int64_t n, const int64_t *rows, const int64_t *cols, double *out)
{
    if (M < 0 || N < 0 || K < 0 || n < 0) return -1;
    if (bad_matrix(A, layoutA, lda, M, K) || bad_matrix(B, layoutB, ldb, K, N)) return -1;
    for (int64_t t = 0; t < n; ++t)
        if (rows[t] < 0 || rows[t] >= M || cols[t] < 0 || cols[t] >= N) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k)
            acc += oracle_bfloat16_bits_to_double(A[at(layoutA, lda, rows[t], k)]) *
                   oracle_bfloat16_bits_to_double(B[at(layoutB, ldb, k, cols[t])]);
        out[t] = acc;
    }
    return 0;
}

/*
 * double -> IEEE 754 binary16 bit pattern, rounded to nearest, ties to even: the single
 * rounding the binary16-output entry point applies to each element of C (the operand
 * types of the paper's executable tensor-core spec, Section 4.2 "Supporting HMMA",
 * have C in FP16).  Written from the format's definition: normal numbers are
 * (1 + f/1024) * 2^(e-15) with 1 <= e <= 30, subnormals f * 2^-24, and a magnitude that
 * rounds to 2^16 or more is infinite.
 */
#include <math.h>
uint16_t oracle_double_to_half_bits(double v)
{
    uint16_t sign = signbit(v) ? 0x8000u : 0u;
    if (isnan(v)) return (uint16_t)(sign | 0x7e00u);
    double a = fabs(v);
    if (isinf(a)) return (uint16_t)(sign | 0x7c00u);
    if (a == 0.0) return sign;
    int ex;
    double m = frexp(a, &ex); /* a = m * 2^ex, 0.5 <= m < 1 */
    int e = ex - 1;           /* a = (2m) * 2^e, 1 <= 2m < 2 */
    if (e < -14) {
        /* subnormal range: multiples of 2^-24; rint rounds to nearest, ties to even */
        double q = rint(ldexp(a, 24));
        return (uint16_t)(sign | (uint16_t)q); /* q == 1024 is the smallest normal number */
    }
    double q = rint(ldexp(2.0 * m - 1.0, 10)); /* fraction in units of 2^-10, 0 .. 1024 */
    if (q == 1024.0) {
        q = 0.0;
        e += 1;
    }
    if (e > 15) return (uint16_t)(sign | 0x7c00u);
    return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)q);
}

/* out[t] = binary16 pattern of in[t], t < n */
int oracle_round_to_half(int64_t n, const double *in, uint16_t *out)
{
    if (n < 0 || (n > 0 && (!in || !out))) return -1;
    for (int64_t t = 0; t < n; ++t) out[t] = oracle_double_to_half_bits(in[t]);
    return 0;
}

/* Number of OpenMP threads the loops above will use (reported with timings). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
