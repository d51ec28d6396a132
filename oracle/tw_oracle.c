/*
 * CPU oracle for the tile-wise (TW) sparse GEMM.  TEST INFRASTRUCTURE ONLY: nothing on the
 * product path may call into this file, and it shares no code with the HIP library.
 *
 * What it computes is the plain definition the method must reach (up to rounding order):
 * the paper turns a product with a TW-pruned weight into several small dense GEMMs
 * (Sec. IV-A, Fig. 4 step 4; Sec. VI first paragraph); the union of those small GEMMs is
 * the masked product
 *
 *      C[m][n] = sum over k with mask[k][n] != 0 of  A[m][k] * B[k][n]
 *
 * with A (M x K) and C (M x N) dense (Sec. VI "Tiling": A and C stay dense, pruned parts
 * are skipped).  Here it is written exactly like that: three nested loops over the mask,
 * no tiles, no index lists, no packing.  Inputs are the 16-bit storage values (fp16 as the
 * paper's tensor-core runs use, Sec. VII-A, or bf16), widened exactly to double; the sum is
 * taken in double, in ascending k.  A column with no kept weight yields exactly 0.
 *
 * two_bias_act is the definition of the fused epilogue (Sec. VI "Kernel Fusion": the bias addition and the
 * activation that follow a weight GEMM): act(C + bias) in double, GELU in its exact form
 * x/2 * (1 + erf(x / sqrt 2)) with the C library's erf.
 *
 * Parity status: pinned (see tests/test_oracle_pins.py): decode tables against numpy/torch,
 * dense special case against BLAS dgemm, closed forms, selector inputs, linearity; two_bias_act
 * against the table value Phi(1), the odd-part identity and hand-made cases.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { TWO_F16 = 0, TWO_BF16 = 1 };

/* IEEE binary16 -> double, exact. */
double two_f16_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int f = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);                 /* zero and subnormals: f * 2^-24 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(f | 0x400), e - 25);    /* (1024+f) * 2^(e-15-10) */
    return sign ? -v : v;
}

/* bfloat16 (upper half of an IEEE binary32) -> double, exact. */
double two_bf16_to_double(uint16_t b)
{
    int sign = (b >> 15) & 1;
    int e = (b >> 7) & 0xFF;
    int f = b & 0x7F;
    double v;
    if (e == 0)
        v = ldexp((double)f, -133);                /* f * 2^-7 * 2^-126 */
    else if (e == 255)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(f | 0x80), e - 134);    /* (128+f) * 2^(e-127-7) */
    return sign ? -v : v;
}

static double widen(uint16_t bits, int dtype)
{
    return dtype == TWO_BF16 ? two_bf16_to_double(bits) : two_f16_to_double(bits);
}

/* Element-wise decode, for the pins. */
int two_decode(const uint16_t *bits, long n, int dtype, double *out)
{
    if (dtype != TWO_F16 && dtype != TWO_BF16) return -1;
    for (long i = 0; i < n; ++i) out[i] = widen(bits[i], dtype);
    return 0;
}

int two_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * C[M x N] (double, row-major, ldc elements) = A . (B masked).
 * A: M x K 16-bit patterns, row-major, lda elements per row.  B: K x N, ldb.  mask: K x N
 * bytes, row-major, N per row, nonzero = kept.  Returns 0, or -1 on a bad argument.
 */
int two_masked_gemm(const uint16_t *A, long lda, const uint16_t *B, long ldb,
                    const uint8_t *mask, long M, long K, long N, int dtype,
                    double *C, long ldc)
{
    if (!A || !B || !mask || !C || M < 0 || K <= 0 || N <= 0) return -1;
    if (lda < K || ldb < N || ldc < N) return -1;
    if (dtype != TWO_F16 && dtype != TWO_BF16) return -1;

    /* widen B once: the same double for every row of A */
    double *Bd = (double *)malloc(sizeof(double) * (size_t)K * (size_t)N);
    if (!Bd) return -2;
    for (long k = 0; k < K; ++k)
        for (long n = 0; n < N; ++n)
            Bd[k * N + n] = widen(B[k * ldb + n], dtype);

#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m) {
        double *c = C + m * ldc;
        for (long n = 0; n < N; ++n) c[n] = 0.0;
        for (long k = 0; k < K; ++k) {                 /* ascending k for every (m, n) */
            double a = widen(A[m * lda + k], dtype);
            const uint8_t *mk = mask + k * N;
            const double *bk = Bd + k * N;
            for (long n = 0; n < N; ++n)
                if (mk[n]) c[n] += a * bk[n];          /* pruned weights are skipped */
        }
    }
    free(Bd);
    return 0;
}

/*
 * In place: C[m][n] = act(C[m][n] + bias[n]) in double; bias may be NULL (no bias).
 * act: 0 none, 1 relu (max(x, 0)), 2 gelu (x/2 * (1 + erf(x / sqrt 2)) = x * Phi(x)).
 * Returns 0, or -1 on a bad argument.
 */
int two_bias_act(double *C, long M, long N, long ldc, const double *bias, int act)
{
    if (!C || M < 0 || N <= 0 || ldc < N || act < 0 || act > 2) return -1;
#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m) {
        double *c = C + m * ldc;
        for (long n = 0; n < N; ++n) {
            double x = c[n] + (bias ? bias[n] : 0.0);
            if (act == 1) x = x > 0.0 ? x : 0.0;
            else if (act == 2) x = 0.5 * x * (1.0 + erf(x / sqrt(2.0)));
            c[n] = x;
        }
    }
    return 0;
}
