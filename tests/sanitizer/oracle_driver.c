/*
 * Runs the CPU oracle's C routines under AddressSanitizer and UndefinedBehaviorSanitizer (built by
 * tests/test_sanitizers.py together with oracle/gemm_oracle.c and oracle/transpose_oracle.c).
 * Every operand sits in a heap block of exactly the bytes its shape and strides span, so a read or write one
 * element outside an operand is reported; expected values are small-integer products worked out by a plain
 * integer triple loop here, so the run also fails on a wrong result.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_gemm_f32(int64_t, int64_t, int64_t, const float *, int64_t, int64_t, const float *, int64_t, int64_t, double *, int64_t, double *, int64_t);
int oracle_gemm_bf16(int64_t, int64_t, int64_t, const uint16_t *, int64_t, int64_t, const uint16_t *, int64_t, int64_t, double *, int64_t, double *, int64_t);
int oracle_gemm_f32_entries(int64_t, const float *, int64_t, int64_t, const float *, int64_t, int64_t, int64_t, const int64_t *, const int64_t *, double *, double *);
int oracle_gemm_bf16_entries(int64_t, const uint16_t *, int64_t, int64_t, const uint16_t *, int64_t, int64_t, int64_t, const int64_t *, const int64_t *, double *, double *);
int oracle_transpose_f32(int64_t, int64_t, const uint32_t *, int64_t, int64_t, uint32_t *, int64_t, int64_t);
void oracle_set_num_threads(int);

static uint64_t state = 12345;
static int small(void) { state = state * 6364136223846793005ull + 1442695040888963407ull; return (int)((state >> 33) % 9) - 4; }
static uint16_t to_bf16(int v) { float f = (float)v; uint32_t w; memcpy(&w, &f, 4); return (uint16_t)(w >> 16); }   /* exact for |v| <= 4 */

#define CHECK(c) do { if (!(c)) { printf("FAILED %s line %d\n", #c, __LINE__); return 1; } } while (0)

/* span of a rows x cols view with the given strides, in elements (0 for an empty view) */
static int64_t span(int64_t rows, int64_t cols, int64_t rs, int64_t cs) { return rows && cols ? (rows - 1) * rs + (cols - 1) * cs + 1 : 0; }

static int one_case(int64_t M, int64_t N, int64_t K, int a_colmajor, int b_colmajor, int64_t pad, int bf16)
{
    const int64_t a_rs = a_colmajor ? 1 : K + pad, a_cs = a_colmajor ? M + pad : 1;
    const int64_t b_rs = b_colmajor ? 1 : N + pad, b_cs = b_colmajor ? K + pad : 1;
    const int64_t na = span(M, K, a_rs, a_cs), nb = span(K, N, b_rs, b_cs), ldc = N + pad, lds = N;
    const size_t es = bf16 ? 2 : 4;
    void *A = malloc(na * es + !na), *B = malloc(nb * es + !nb);
    double *C = malloc(sizeof(double) * (size_t)(M ? (M - 1) * ldc + N : 0) + 8), *S = malloc(sizeof(double) * (size_t)(M * lds) + 8);
    int *ia = calloc((size_t)(M * K) + 1, sizeof(int)), *ib = calloc((size_t)(K * N) + 1, sizeof(int));
    memset(A, 0xFF, na * es), memset(B, 0xFF, nb * es);      /* padding holds NaN patterns */
    for (int64_t i = 0; i < M; ++i)
        for (int64_t k = 0; k < K; ++k) {
            const int v = small();
            ia[i * K + k] = v;
            if (bf16) ((uint16_t *)A)[i * a_rs + k * a_cs] = to_bf16(v); else ((float *)A)[i * a_rs + k * a_cs] = (float)v;
        }
    for (int64_t k = 0; k < K; ++k)
        for (int64_t j = 0; j < N; ++j) {
            const int v = small();
            ib[k * N + j] = v;
            if (bf16) ((uint16_t *)B)[k * b_rs + j * b_cs] = to_bf16(v); else ((float *)B)[k * b_rs + j * b_cs] = (float)v;
        }
    int rc = bf16 ? oracle_gemm_bf16(M, N, K, A, a_rs, a_cs, B, b_rs, b_cs, C, ldc, S, lds)
                  : oracle_gemm_f32(M, N, K, A, a_rs, a_cs, B, b_rs, b_cs, C, ldc, S, lds);
    CHECK(rc == 0);
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            long want = 0, mag = 0;
            for (int64_t k = 0; k < K; ++k) want += ia[i * K + k] * ib[k * N + j], mag += labs((long)ia[i * K + k] * ib[k * N + j]);
            CHECK(C[i * ldc + j] == (double)want && S[i * lds + j] == (double)mag);
        }
    if (M && N) {       /* the entries-only routine on the corners and a middle entry, with and without the scale */
        int64_t ii[3] = {0, M - 1, M / 2}, jj[3] = {N - 1, 0, N / 2};
        double c[3], s[3];
        rc = bf16 ? oracle_gemm_bf16_entries(K, A, a_rs, a_cs, B, b_rs, b_cs, 3, ii, jj, c, s) : oracle_gemm_f32_entries(K, A, a_rs, a_cs, B, b_rs, b_cs, 3, ii, jj, c, s);
        CHECK(rc == 0);
        for (int t = 0; t < 3; ++t) CHECK(c[t] == C[ii[t] * ldc + jj[t]] && s[t] == S[ii[t] * lds + jj[t]]);
        rc = bf16 ? oracle_gemm_bf16_entries(K, A, a_rs, a_cs, B, b_rs, b_cs, 3, ii, jj, c, NULL) : oracle_gemm_f32_entries(K, A, a_rs, a_cs, B, b_rs, b_cs, 3, ii, jj, c, NULL);
        CHECK(rc == 0 && c[0] == C[ii[0] * ldc + jj[0]]);
    }
    /* without the scale */
    rc = bf16 ? oracle_gemm_bf16(M, N, K, A, a_rs, a_cs, B, b_rs, b_cs, C, ldc, NULL, 0) : oracle_gemm_f32(M, N, K, A, a_rs, a_cs, B, b_rs, b_cs, C, ldc, NULL, 0);
    CHECK(rc == 0);
    free(A), free(B), free(C), free(S), free(ia), free(ib);
    return 0;
}

static int transposes(void)
{
    const int64_t shapes[][2] = {{1, 1}, {1, 7}, {7, 1}, {5, 3}, {64, 65}, {33, 130}, {0, 4}, {4, 0}};
    for (size_t t = 0; t < sizeof shapes / sizeof shapes[0]; ++t)
        for (int64_t pad = 0; pad < 3; ++pad) {
            const int64_t r = shapes[t][0], c = shapes[t][1], lda = c + pad, ldt = r + 2 * pad;
            uint32_t *A = malloc(4 * (size_t)span(r, c, lda, 1) + 4), *T = malloc(4 * (size_t)span(c, r, ldt, 1) + 4);
            for (int64_t i = 0; i < r; ++i) for (int64_t j = 0; j < c; ++j) A[i * lda + j] = (uint32_t)(i * 1000003 + j * 7 + 0x7FC00001u);   /* NaN payloads too */
            CHECK(oracle_transpose_f32(r, c, A, lda, 1, T, ldt, 1) == 0);
            for (int64_t i = 0; i < r; ++i) for (int64_t j = 0; j < c; ++j) CHECK(T[j * ldt + i] == A[i * lda + j]);
            free(A), free(T);
        }
    CHECK(oracle_transpose_f32(-1, 3, NULL, 1, 1, NULL, 1, 1) != 0);
    return 0;
}

int main(void)
{
    const int64_t dims[] = {0, 1, 2, 3, 5, 17, 33};
    const int nd = (int)(sizeof dims / sizeof dims[0]);
    int cases = 0;
    for (int threads = 1; threads <= 4; threads += 3) {
        oracle_set_num_threads(threads);
        for (int a = 0; a < nd; ++a) for (int b = 0; b < nd; ++b) for (int c = 0; c < nd; ++c)
            for (int lay = 0; lay < 4; ++lay) for (int bf16 = 0; bf16 < 2; ++bf16) {
                if (one_case(dims[a], dims[b], dims[c], lay & 1, lay >> 1, (a + b + c) % 3, bf16)) return 1;
                ++cases;
            }
    }
    if (one_case(70, 90, 300, 0, 1, 5, 0) || one_case(70, 90, 300, 1, 0, 0, 1)) return 1;
    if (transposes()) return 1;
    printf("oracle under sanitizers: %d product cases and the transposes ok\n", cases + 2);
    return 0;
}
