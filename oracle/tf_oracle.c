/*
 * CPU oracle for the fused tile kernel  Y = GELU_erf(A.B + bias) (B as [K][N], or as [N][K] in
 * tfo_gemm_nt_bias_gelu), and (last two functions of
 * the file but one) for the batched vector-matrix product of the paper's Case Study 2 and the
 * batched transposed-operand product of its Case Study 3, and (last) for the element-wise sine of
 * its Case Study 1.  tfo_gelu_tanh is the activation of the kernel's second bf16 epilogue.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU kernels are checked against.  It is single-threaded, has no blocking,
 * no SIMD intrinsics and no BLAS, and shares no code, header, table or helper
 * with the HIP library.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the product never does.
 *
 * What is computed (the kernel is the tile-level kernel that the paper's
 * profile -> analyse -> transform -> evaluate loop of Sec. 3.3 / Algorithm 1
 * treats as its input K; its arithmetic is fixed by the workload definition,
 * not by the paper, which prints no formula for it):
 *
 *   z[m,n] = sum_{k=0}^{K-1} a[m,k] * b[k,n] + bias[n]
 *   y[m,n] = GELU(z) = 1/2 * z * (1 + erf(z / sqrt 2))
 *   s[m,n] = sum_k |a[m,k] * b[k,n]| + |bias[n]|      (for a-priori error bounds)
 *
 * a, b, bias are the exact real values of the bf16 bit patterns handed in.
 * All arithmetic is IEEE double: a product of two bf16 values has at most 16
 * significand bits and is exact in double, so only the running sum rounds.
 * Layouts are row-major with leading dimensions in elements: A[M,K] (lda),
 * B[K,N] (ldb), bias[N]; outputs are dense M x N doubles (ld = N).
 *
 * Every function here is pinned by tests that do not call back into this file
 * to produce the expected value: exact rational brute force on tiny inputs,
 * closed-form GELU values x*Phi(x), the identity GELU(x) - GELU(-x) = x,
 * identity / zero / ones / rank-1 operands, exact power-of-two scaling,
 * integer-valued operands, and numpy's float64 matmul.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#include <stdlib.h>

/* bf16 is the upper half of an IEEE binary32: widen by appending 16 zero bits. */
double tfo_bf16_to_double(uint16_t bits)
{
    uint32_t w = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* Exact-erf GELU, x * Phi(x).  For negative x the factor (1 + erf) cancels, so
 * the same quantity is written with erfc:  1 + erf(t) = erfc(-t). */
double tfo_gelu(double z)
{
    const double inv_sqrt2 = 0.70710678118654752440;
    if (z < 0.0)
        return 0.5 * z * erfc(-z * inv_sqrt2);
    return 0.5 * z * (1.0 + erf(z * inv_sqrt2));
}

/* The tanh form of GELU (Hendrycks and Gimpel's approximation, the other activation the epilogue
 * offers):  1/2 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3))), written out with libm's tanh.
 * Pinned by tests/test_oracle_gemm.py: 50-digit decimal evaluation through exp, the odd-part
 * identity, limits, and its known distance from the erf form. */
double tfo_gelu_tanh(double z)
{
    const double c = 0.79788456080286535588; /* sqrt(2/pi) */
    return 0.5 * z * (1.0 + tanh(c * (z + 0.044715 * z * z * z)));
}

/* y[i] = tfo_gelu_tanh(z[i]) for i < n.  Returns 0, or -1 on a bad argument. */
int tfo_gelu_tanh_array(long n, const double *z, double *y)
{
    if (n < 0 || (n > 0 && (!z || !y)))
        return -1;
    for (long i = 0; i < n; ++i)
        y[i] = tfo_gelu_tanh(z[i]);
    return 0;
}

/*
 * Full problem.  Any of Y, Z, S may be NULL (not wanted).
 * Returns 0, or -1 on a bad argument, -2 if the row buffers cannot be allocated.
 * Loop order is i, k, j with one row of accumulators: still the plain triple
 * loop, each z[m,n] is summed in increasing k.
 */
int tfo_gemm_bias_gelu(int M, int N, int K,
                       const uint16_t *A, long lda,
                       const uint16_t *B, long ldb,
                       const uint16_t *bias,
                       double *Y, double *Z, double *S)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if (M == 0 || N == 0) return 0;
    if ((K > 0 && (!A || !B)) || !bias) return -1;
    if (lda < K || ldb < N) return -1;

    double *acc = (double *)malloc(sizeof(double) * (size_t)N);
    double *abs_acc = (double *)malloc(sizeof(double) * (size_t)N);
    if (!acc || !abs_acc) { free(acc); free(abs_acc); return -2; }

    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) { acc[n] = 0.0; abs_acc[n] = 0.0; }
        for (int k = 0; k < K; ++k) {
            const double a = tfo_bf16_to_double(A[(size_t)m * (size_t)lda + (size_t)k]);
            const uint16_t *brow = B + (size_t)k * (size_t)ldb;
            for (int n = 0; n < N; ++n) {
                const double p = a * tfo_bf16_to_double(brow[n]);
                acc[n] += p;
                abs_acc[n] += fabs(p);
            }
        }
        for (int n = 0; n < N; ++n) {
            const double bv = tfo_bf16_to_double(bias[n]);
            const double z = acc[n] + bv;
            const size_t o = (size_t)m * (size_t)N + (size_t)n;
            if (Z) Z[o] = z;
            if (Y) Y[o] = tfo_gelu(z);
            if (S) S[o] = abs_acc[n] + fabs(bv);
        }
    }
    free(acc);
    free(abs_acc);
    return 0;
}

/*
 * Selected outputs only: for each t < count, the element (rows[t], cols[t]),
 * written out as the dot product of one row of A with one column of B.
 * Used where the whole problem is too large to evaluate on the host.
 */
int tfo_gemm_bias_gelu_at(int M, int N, int K,
                          const uint16_t *A, long lda,
                          const uint16_t *B, long ldb,
                          const uint16_t *bias,
                          long count, const int *rows, const int *cols,
                          double *y, double *z, double *s)
{
    if (M < 0 || N < 0 || K < 0 || count < 0) return -1;
    if (count > 0 && (!rows || !cols || !bias)) return -1;
    if (K > 0 && count > 0 && (!A || !B)) return -1;
    if (lda < K || ldb < N) return -1;
    for (long t = 0; t < count; ++t) {
        const int m = rows[t], n = cols[t];
        if (m < 0 || m >= M || n < 0 || n >= N) return -1;
        double acc = 0.0, abs_acc = 0.0;
        for (int k = 0; k < K; ++k) {
            const double p = tfo_bf16_to_double(A[(size_t)m * (size_t)lda + (size_t)k]) *
                             tfo_bf16_to_double(B[(size_t)k * (size_t)ldb + (size_t)n]);
            acc += p;
            abs_acc += fabs(p);
        }
        const double bv = tfo_bf16_to_double(bias[n]);
        const double zz = acc + bv;
        if (z) z[t] = zz;
        if (y) y[t] = tfo_gelu(zz);
        if (s) s[t] = abs_acc + fabs(bv);
    }
    return 0;
}

/*
 * The same operation with the second operand given as [N][ldb], k contiguous (a weight matrix
 * stored output-major; the layout question of the paper's Case Study 3, where an operand arrives
 * transposed and the kernel either reads it as it lies or pays for a separate transposing pass):
 *     z[m,n] = sum_{k=0}^{K-1} a[m,k] * bt[n,k] + bias[n],   y = GELU(z),   s = sum |a bt| + |bias|
 * Written out as the definition: three nested loops (m, n, k), one dot product of two rows per
 * element, products and sums in double, k ascending. Any of Y, Z, S may be NULL.
 * Pinned by tests/test_oracle_gemm_nt.py: exact rational brute force, selector matrices that
 * copy single columns of A, integer operands against an int64 contraction, a library product
 * of the explicitly transposed operand, power-of-two scaling, and the zero-matrix / GELU(0)
 * cases.
 */
int tfo_gemm_nt_bias_gelu(int M, int N, int K,
                          const uint16_t *A, long lda,
                          const uint16_t *Bt, long ldb,
                          const uint16_t *bias,
                          double *Y, double *Z, double *S)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if (M == 0 || N == 0) return 0;
    if ((K > 0 && (!A || !Bt)) || !bias) return -1;
    if (lda < K || ldb < K) return -1;
    for (int m = 0; m < M; ++m) {
        const uint16_t *arow = A + (size_t)m * (size_t)lda;
        for (int n = 0; n < N; ++n) {
            const uint16_t *brow = Bt + (size_t)n * (size_t)ldb;
            double acc = 0.0, abs_acc = 0.0;
            for (int k = 0; k < K; ++k) {
                const double p = tfo_bf16_to_double(arow[k]) * tfo_bf16_to_double(brow[k]);
                acc += p;
                abs_acc += fabs(p);
            }
            const double bv = tfo_bf16_to_double(bias[n]);
            const double z = acc + bv;
            const size_t o = (size_t)m * (size_t)N + (size_t)n;
            if (Z) Z[o] = z;
            if (Y) Y[o] = tfo_gelu(z);
            if (S) S[o] = abs_acc + fabs(bv);
        }
    }
    return 0;
}

/*
 * Batched vector-matrix product of the paper's Case Study 2:
 *     C[m][n] = sum_{k=0}^{K-1} A[m][k] * B[m][n][k]
 * A is [M][lda] (lda >= K), B is [M][N][ldb] (ldb >= K, k contiguous, the matrices of the batch
 * one after the other), all bf16 bit patterns; C and S are [M][N] doubles (S = sum |a b|, the
 * scale of a rounding-error bound; may be NULL). The definition written out: three nested
 * loops, products and sums in double, k ascending.
 * Pinned by tests/test_oracle_bvm.py: exact rational arithmetic on small cases, A = ones (row
 * sums of B by an independent exactly rounded summation), a Kronecker-delta B that picks single
 * elements of A, the one-row case against a library matrix-vector product, integer operands,
 * power-of-two scaling.
 */
int tfo_batched_vecmat(int M, int N, int K,
                       const uint16_t *A, long lda,
                       const uint16_t *B, long ldb,
                       double *C, double *S)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if (lda < K || ldb < K) return -1;
    if (M > 0 && N > 0 && !C) return -1;
    if (M > 0 && N > 0 && K > 0 && (!A || !B)) return -1;
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            const uint16_t *brow = B + ((size_t)m * (size_t)N + (size_t)n) * (size_t)ldb;
            double acc = 0.0, abs_acc = 0.0;
            for (int k = 0; k < K; ++k) {
                const double p = tfo_bf16_to_double(A[(size_t)m * (size_t)lda + (size_t)k]) *
                                 tfo_bf16_to_double(brow[k]);
                acc += p;
                abs_acc += fabs(p);
            }
            C[(size_t)m * (size_t)N + (size_t)n] = acc;
            if (S) S[(size_t)m * (size_t)N + (size_t)n] = abs_acc;
        }
    }
    return 0;
}

/*
 * Batched product with the first operand given transposed, the gradient term of the paper's
 * Case Study 3 (dB = dO^T A, one product per chunk):
 *     C[b][m][n] = sum_{k=0}^{K-1} A[b][k][m] * B[b][k][n]
 * A[b] is [K][lda] (lda >= M, m contiguous), B[b] is [K][ldb] (ldb >= N), consecutive batch
 * items stride_a resp. stride_b elements apart; all bf16 bit patterns. C and S (sum |a b|, may
 * be NULL) are dense [batch][M][N] doubles. Four nested loops, k ascending, sums in double.
 * Pinned by tests/test_oracle_bgemm.py: exact rational arithmetic, selector matrices that copy
 * single rows of B, integer operands against an int64 contraction, the one-item case against a
 * library matrix product of the explicitly transposed operand, power-of-two scaling, batch
 * independence.
 */
int tfo_batched_gemm_tn(int batch, int M, int N, int K,
                        const uint16_t *A, long lda, long stride_a,
                        const uint16_t *B, long ldb, long stride_b,
                        double *C, double *S)
{
    if (batch < 0 || M < 0 || N < 0 || K < 0) return -1;
    if (lda < M || ldb < N) return -1;
    if (batch > 0 && M > 0 && N > 0 && !C) return -1;
    if (batch > 0 && M > 0 && N > 0 && K > 0 && (!A || !B)) return -1;
    for (int b = 0; b < batch; ++b) {
        const uint16_t *Ab = A + (size_t)b * (size_t)stride_a;
        const uint16_t *Bb = B + (size_t)b * (size_t)stride_b;
        for (int m = 0; m < M; ++m) {
            for (int n = 0; n < N; ++n) {
                double acc = 0.0, abs_acc = 0.0;
                for (int k = 0; k < K; ++k) {
                    const double p = tfo_bf16_to_double(Ab[(size_t)k * (size_t)lda + (size_t)m]) *
                                     tfo_bf16_to_double(Bb[(size_t)k * (size_t)ldb + (size_t)n]);
                    acc += p;
                    abs_acc += fabs(p);
                }
                const size_t o = ((size_t)b * (size_t)M + (size_t)m) * (size_t)N + (size_t)n;
                C[o] = acc;
                if (S) S[o] = abs_acc;
            }
        }
    }
    return 0;
}

/*
 * Element-wise sine of the paper's Case Study 1 (a kernel whose only tuning axis is the launch
 * shape):  y[i] = sin(x[i]),  x given as IEEE binary32 values, evaluated in double by libm.
 * Pinned by tests/test_oracle_sin.py: exact rational Taylor sums of the binary32 inputs, odd
 * symmetry, exact zeros, the bound |y| <= 1, and multiples of pi rounded to binary32 against
 * the first-order expansion around the true multiple.
 */
int tfo_sin_f32(long n, const float *x, double *y)
{
    if (n < 0) return -1;
    if (n > 0 && (!x || !y)) return -1;
    for (long i = 0; i < n; ++i) y[i] = sin((double)x[i]);
    return 0;
}
