/*
 * CPU oracle for dense matrix multiplication C = A x B (the paper's Task 2
 * definition in its task-prompt table: A is M x K, B is K x N, C is M x N).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the GPU library includes, links or
 * calls this file; it shares no header, helper or constant with it.
 *
 * The definition is written out directly:
 *
 *     C[i][j] = sum_{k=0}^{K-1} (double)A[i][k] * (double)B[k][j]
 *
 * accumulated in fp64 in increasing k.  For fp32 or bf16 inputs every
 * product is exact in fp64 (24+24 <= 53 significand bits), so only the K-1
 * additions round.  Alongside C the oracle can return the magnitude sum
 *
 *     S[i][j] = sum_k |A[i][k]| * |B[k][j]|
 *
 * which is the scale of the standard componentwise error bound for a dot
 * product and is what tolerances are measured against.
 *
 * Operands are addressed through explicit (row stride, column stride) pairs
 * in elements, so row-major, column-major and padded leading dimensions all
 * go through the same loop.  The loop nest is i, k, j with a per-row fp64
 * accumulator: each C[i][j] still receives its K terms in increasing k.
 * OpenMP splits rows i only, so no sum is ever divided between threads and
 * the result does not depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* bf16 -> fp32 is exact: the 16 bits are the top half of the IEEE-754 word. */
static inline float bf16_bits_to_float(uint16_t h)
{
    uint32_t w = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return f;
}

#define ORACLE_GEMM_BODY(LOAD_A, LOAD_B)                                       \
    if (M <= 0 || N <= 0) return 0;                                            \
    _Pragma("omp parallel")                                                    \
    {                                                                          \
        double *acc = (double *)malloc(sizeof(double) * (size_t)N);            \
        double *mag = (double *)malloc(sizeof(double) * (size_t)N);            \
        _Pragma("omp for schedule(static)")                                    \
        for (int64_t i = 0; i < M; ++i) {                                      \
            for (int64_t j = 0; j < N; ++j) { acc[j] = 0.0; mag[j] = 0.0; }    \
            for (int64_t k = 0; k < K; ++k) {                                  \
                const double a = (double)LOAD_A(A[i * a_rs + k * a_cs]);       \
                const double fa = fabs(a);                                     \
                for (int64_t j = 0; j < N; ++j) {                              \
                    const double b = (double)LOAD_B(B[k * b_rs + j * b_cs]);   \
                    acc[j] += a * b;                                           \
                    mag[j] += fa * fabs(b);                                    \
                }                                                              \
            }                                                                  \
            for (int64_t j = 0; j < N; ++j) C[i * ldc + j] = acc[j];           \
            if (S) for (int64_t j = 0; j < N; ++j) S[i * lds + j] = mag[j];    \
        }                                                                      \
        free(acc);                                                             \
        free(mag);                                                             \
    }                                                                          \
    return 0;

#define IDENT(x) (x)

/* fp32 operands; C and S (S may be NULL) are row-major fp64 with leading
 * dimensions ldc / lds.  Host pointers. */
int oracle_gemm_f32(int64_t M, int64_t N, int64_t K,
                    const float *A, int64_t a_rs, int64_t a_cs,
                    const float *B, int64_t b_rs, int64_t b_cs,
                    double *C, int64_t ldc, double *S, int64_t lds)
{
    ORACLE_GEMM_BODY(IDENT, IDENT)
}

/* bf16 operands given as raw 16-bit patterns. */
int oracle_gemm_bf16(int64_t M, int64_t N, int64_t K,
                     const uint16_t *A, int64_t a_rs, int64_t a_cs,
                     const uint16_t *B, int64_t b_rs, int64_t b_cs,
                     double *C, int64_t ldc, double *S, int64_t lds)
{
    ORACLE_GEMM_BODY(bf16_bits_to_float, bf16_bits_to_float)
}

/* Selected entries only: for t in [0, n) compute C[ii[t]][jj[t]] and the
 * matching S, each by the same increasing-k fp64 sum.  Used where the full
 * product is too large for the CPU. */
int oracle_gemm_f32_entries(int64_t K,
                            const float *A, int64_t a_rs, int64_t a_cs,
                            const float *B, int64_t b_rs, int64_t b_cs,
                            int64_t n, const int64_t *ii, const int64_t *jj,
                            double *c_out, double *s_out)
{
    #pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        const int64_t i = ii[t], j = jj[t];
        double acc = 0.0, mag = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = (double)A[i * a_rs + k * a_cs];
            const double b = (double)B[k * b_rs + j * b_cs];
            acc += a * b;
            mag += fabs(a) * fabs(b);
        }
        c_out[t] = acc;
        if (s_out) s_out[t] = mag;
    }
    return 0;
}

int oracle_gemm_bf16_entries(int64_t K,
                             const uint16_t *A, int64_t a_rs, int64_t a_cs,
                             const uint16_t *B, int64_t b_rs, int64_t b_cs,
                             int64_t n, const int64_t *ii, const int64_t *jj,
                             double *c_out, double *s_out)
{
    #pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        const int64_t i = ii[t], j = jj[t];
        double acc = 0.0, mag = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = (double)bf16_bits_to_float(A[i * a_rs + k * a_cs]);
            const double b = (double)bf16_bits_to_float(B[k * b_rs + j * b_cs]);
            acc += a * b;
            mag += fabs(a) * fabs(b);
        }
        c_out[t] = acc;
        if (s_out) s_out[t] = mag;
    }
    return 0;
}

/* Threads the row loop will use (1 without OpenMP). */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
