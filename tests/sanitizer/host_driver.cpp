// Runs the host side of the C ABI -- argument checks, plans, kernel names, workspace sizes -- under AddressSanitizer
// and UndefinedBehaviorSanitizer (tests/test_sanitizers.py compiles csrc/api.hip with the sanitizers on its host
// pass and links it with this file and the library's other objects).  Only queries and calls that are rejected
// before any launch are made: the addresses are fake, so nothing here may reach a kernel.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "fsrgemm.h"

#define CHECK(c) do { if (!(c)) { printf("FAILED %s line %d\n", #c, __LINE__); return 1; } } while (0)

static uint64_t state = 99;
static uint64_t next() { state = state * 6364136223846793005ull + 1442695040888963407ull; return state >> 33; }
template <class T, size_t N> static T pick(const T (&a)[N]) { return a[next() % N]; }

int main()
{
    const int64_t dims[] = {0, 1, 2, 7, 10, 16, 17, 63, 64, 65, 255, 256, 257, 1000, 2048, 2560, 3072, 4096, 4097, 5120, 8192, 1 << 16, 1 << 20, (1 << 22) + 3, (1ll << 31) - 1};
    const int64_t pads[] = {0, 0, 1, 3, 4, 8, 1 << 24, 1ll << 25, 1ll << 31};
    const uintptr_t offs[] = {0, 0, 1, 2, 4};
    const uintptr_t P = 0x1000;
    const int n32 = fsrgemm_tile_count_f32(), n16 = fsrgemm_tile_count_bf16();
    CHECK(n32 == 17 && n16 == 11 && fsrgemm_version() >= 200);
    long plans = 0, names = 0;
    for (int c = 0; c < 20000; ++c) {
        const int ta = (int)(next() & 1), tb = (int)(next() & 1);
        int64_t M = pick(dims), N = pick(dims), K = pick(dims);
        const int64_t lda = (ta ? M : K) + pick(pads), ldb = (tb ? K : N) + pick(pads), ldc = N + (int64_t)(next() % 5);
        for (int bf16 = 0; bf16 < 2; ++bf16) {
            const uintptr_t es = bf16 ? 2 : 4;
            const void *a = (const void *)(P + es * pick(offs)), *b = (const void *)(P + es * pick(offs));
            const float *cptr = (const float *)P;
            for (int flags = 0; flags < 4; ++flags) {
                int tile = -7, slices = -7;
                const int rc = bf16 ? fsrgemm_plan_bf16(ta, tb, M, N, K, (const uint16_t *)a, lda, (const uint16_t *)b, ldb, flags, &tile, &slices)
                                    : fsrgemm_plan_f32(ta, tb, M, N, K, (const float *)a, lda, (const float *)b, ldb, flags, &tile, &slices);
                if (rc != FSRGEMM_OK) continue;
                ++plans;
                CHECK(tile >= 0 && tile < (bf16 ? n16 : n32) && slices >= 1 && slices <= 256);
                // the same plan in terms of bands: one launch, or a cut at a multiple of 64 strictly inside C
                int dim = -7, first = -7, second = -7;
                int64_t at = -7;
                CHECK((bf16 ? fsrgemm_bands_bf16(ta, tb, M, N, K, (const uint16_t *)a, lda, (const uint16_t *)b, ldb, flags, &dim, &at, &first, &second)
                            : fsrgemm_bands_f32(ta, tb, M, N, K, (const float *)a, lda, (const float *)b, ldb, flags, &dim, &at, &first, &second)) == FSRGEMM_OK);
                CHECK(first == tile && second >= 0 && second < (bf16 ? n16 : n32));
                CHECK(dim == 0 ? (at == 0 && second == first) : ((dim == 1 || dim == 2) && at % 64 == 0 && at > 0 && at < (dim == 1 ? M : N) && slices == 1));
                if (M > 0 && N > 0 && M * N < (1ll << 40)) {
                    const char *nm = bf16 ? fsrgemm_kernel_for_bf16_cfg(tile, ta, tb, M, N, K, (const uint16_t *)a, lda, (const uint16_t *)b, ldb, cptr, ldc)
                                          : fsrgemm_kernel_for_f32_cfg(tile, ta, tb, M, N, K, (const float *)a, lda, (const float *)b, ldb, cptr, ldc);
                    CHECK(nm != nullptr && strlen(nm) > 8);
                    ++names;
                }
            }
            const int64_t ws = bf16 ? gemm_bf16_workspace_bytes(ta, tb, M, N, K) : gemm_f32_workspace_bytes(ta, tb, M, N, K);
            CHECK(ws >= 0 && ws <= (16 << 20));
            const char *nm = bf16 ? fsrgemm_kernel_for_bf16_ex(ta, tb, M, N, K, (const uint16_t *)a, lda, (const uint16_t *)b, ldb, cptr, ldc)
                                  : fsrgemm_kernel_for_f32_ex(ta, tb, M, N, K, (const float *)a, lda, (const float *)b, ldb, cptr, ldc);
            (void)nm;
            // every forced candidate: a name or NULL, never a crash
            for (int tile = -1; tile <= (bf16 ? n16 : n32); ++tile) {
                const char *fn = bf16 ? fsrgemm_kernel_for_bf16_cfg(tile, ta, tb, M, N, K, (const uint16_t *)a, lda, (const uint16_t *)b, ldb, cptr, ldc)
                                      : fsrgemm_kernel_for_f32_cfg(tile, ta, tb, M, N, K, (const float *)a, lda, (const float *)b, ldb, cptr, ldc);
                if (fn) ++names;
            }
            // calls that the argument checks reject: a negative extent, a leading dimension one short, a missing C
            CHECK((bf16 ? gemm_bf16_ex(ta, tb, -1, N, K, (const uint16_t *)a, lda, (const uint16_t *)b, ldb, (float *)P, ldc, nullptr)
                        : gemm_f32_ex(ta, tb, -1, N, K, (const float *)a, lda, (const float *)b, ldb, (float *)P, ldc, nullptr)) == FSRGEMM_ERR_INVALID_ARG);
            if (M > 0 && N > 0) {
                CHECK((bf16 ? gemm_bf16_ws(ta, tb, M, N, K, (const uint16_t *)a, lda, (const uint16_t *)b, ldb, nullptr, ldc, nullptr, 0, nullptr)
                            : gemm_f32_ws(ta, tb, M, N, K, (const float *)a, lda, (const float *)b, ldb, nullptr, ldc, nullptr, 0, nullptr)) == FSRGEMM_ERR_INVALID_ARG);
                CHECK((bf16 ? gemm_bf16_cfg(0, 1, ta, tb, M, N, K, (const uint16_t *)a, lda, (const uint16_t *)b, ldb, (float *)P, N - 1, nullptr, 0, nullptr)
                            : gemm_f32_cfg(0, 1, ta, tb, M, N, K, (const float *)a, lda, (const float *)b, ldb, (float *)P, N - 1, nullptr, 0, nullptr)) == FSRGEMM_ERR_INVALID_ARG);
                if (!bf16) CHECK(gemm_f32_noalloc(ta, tb, M, N, K, (const float *)a, lda, (const float *)b, ldb, nullptr, ldc, nullptr) == FSRGEMM_ERR_INVALID_ARG);
            }
        }
        const int64_t r = pick(dims), q = pick(dims);
        const char *tn = fsrgemm_kernel_for_transpose_f32(r, q, (const float *)P, q + (int64_t)(next() % 3), (const float *)P, r + (int64_t)(next() % 3));
        (void)tn;
        CHECK(transpose_f32(r, q, (const float *)P, q - 1, (float *)P, r, nullptr) == FSRGEMM_ERR_INVALID_ARG || q == 0);
    }
    double flop = 0;
    CHECK(fsrgemm_mfma_ceiling(2, 1, (const void *)P, (float *)P, 1, &flop, nullptr) == FSRGEMM_ERR_INVALID_ARG);
    CHECK(fsrgemm_kernel_for_mfma_ceiling(0) && fsrgemm_kernel_for_mfma_ceiling(1) && !fsrgemm_kernel_for_mfma_ceiling(-1));
    for (int s = -6; s <= 1; ++s) CHECK(fsrgemm_status_string(s) != nullptr);
    printf("host dispatch under sanitizers: %ld plans, %ld kernel names ok\n", plans, names);
    return 0;
}
