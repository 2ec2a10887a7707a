// C ABI of the library (declared in include/fsrgemm.h): argument checks,
// choice of tile configuration and load mode, launch on the caller's stream.
#include "../../include/fsrgemm.h"

#include <string.h>

#include "common.hpp"

using namespace fsrgemm;

namespace {

struct Plan {
    int cfg;
    int mode;
};

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks shared by all entry points.  lda_min / ldb_min are the extents of the operands' contiguous index (K or M
// for A, N or K for B, by storage order).  Returns FSRGEMM_OK when the problem is well formed.
int check_args(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, int64_t lda_min, const void *B,
               int64_t ldb, int64_t ldb_min, const void *C, int64_t ldc)
{
    const int64_t lim = (int64_t)1 << 31;
    if (M < 0 || N < 0 || K < 0 || M >= lim || N >= lim || K >= lim) return FSRGEMM_ERR_INVALID_ARG;
    if (lda < lda_min || ldb < ldb_min || ldc < N) return FSRGEMM_ERR_INVALID_ARG;
    if (M > 0 && N > 0 && C == nullptr) return FSRGEMM_ERR_INVALID_ARG;
    if (M > 0 && N > 0 && K > 0 && (A == nullptr || B == nullptr)) return FSRGEMM_ERR_INVALID_ARG;
    return FSRGEMM_OK;
}

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// The largest tile whose grid still fills the chip (256 compute units, two or more workgroups each for the
// smaller tiles); the load mode follows from alignment and divisibility.  Grids beyond 2^31 - 1 workgroups are
// rejected.
int plan_f32(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb, Plan *p)
{
    int bm, bn;
    if (ceil_div(M, 256) * ceil_div(N, 128) >= 384) p->cfg = kF32_256x128, bm = 256, bn = 128;
    else if (ceil_div(M, 128) * ceil_div(N, 128) >= 256) p->cfg = kF32_128x128, bm = 128, bn = 128;
    else p->cfg = kF32_64x64, bm = 64, bn = 64;
    if (ceil_div(M, bm) * ceil_div(N, bn) >= ((int64_t)1 << 31)) return FSRGEMM_ERR_INVALID_ARG;
    const bool vec = aligned16(A) && aligned16(B) && lda % 4 == 0 && ldb % 4 == 0;
    // unchecked loads and stores need whole K-tiles and a matrix at least one tile wide and high (a ragged last
    // tile is shifted back into the matrix)
    p->mode = !vec ? kScalar : (M >= bm && N >= bn && K % 16 == 0 && K > 0) ? kFast : kVecPred;
    return FSRGEMM_OK;
}

int plan_bf16(int a_lay, int b_lay, int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda, const uint16_t *B,
              int64_t ldb, Plan *p)
{
    int b;
    if (ceil_div(M, 256) * ceil_div(N, 256) >= 128) p->cfg = kBf16_256x256, b = 256;
    else if (ceil_div(M, 128) * ceil_div(N, 128) >= 256) p->cfg = kBf16_128x128, b = 128;
    else p->cfg = kBf16_64x64, b = 64;
    if (ceil_div(M, b) * ceil_div(N, b) >= ((int64_t)1 << 31)) return FSRGEMM_ERR_INVALID_ARG;
    const bool vec = aligned16(A) && aligned16(B) && lda % 8 == 0 && ldb % 8 == 0;
    p->mode = !vec ? kScalar : (M >= b && N >= b && K % 64 == 0 && K > 0) ? kFast : kVecPred;
    // the direct-to-LDS kernel needs unchecked 256 x 256 x 64 tiles, 32-bit lane offsets and, for an operand
    // that is contiguous along m (n), M (N) a multiple of 8: a shifted last tile must still start 16-byte aligned
    if (b == 256 && p->mode == kFast && lda < (1 << 25) && ldb < (1 << 25) && (a_lay == kKContig || M % 8 == 0) &&
        (b_lay == kKContig || N % 8 == 0))
        p->cfg = kBf16_Main;
    return FSRGEMM_OK;
}

// gfx950 check for the current device, cached per device ordinal (racing first calls just repeat the query).
int device_ok()
{
    constexpr int kMaxDev = 64;
    static std::atomic<int> cache[kMaxDev];     // 0 = unknown, 1 = gfx950, 2 = something else
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return FSRGEMM_ERR_UNSUPPORTED_DEVICE;
    const bool cached = dev >= 0 && dev < kMaxDev;
    if (cached) {
        const int c = cache[dev].load(std::memory_order_relaxed);
        if (c) return c == 1 ? FSRGEMM_OK : FSRGEMM_ERR_UNSUPPORTED_DEVICE;
    }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return FSRGEMM_ERR_UNSUPPORTED_DEVICE;
    const bool ok = strncmp(prop.gcnArchName, "gfx950", 6) == 0;
    if (cached) cache[dev].store(ok ? 1 : 2, std::memory_order_relaxed);
    return ok ? FSRGEMM_OK : FSRGEMM_ERR_UNSUPPORTED_DEVICE;
}

GemmArgs pack(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb, float *C,
              int64_t ldc)
{
    GemmArgs a;
    a.M = (int)M;
    a.N = (int)N;
    a.K = (int)K;
    a.A = A;
    a.lda = lda;
    a.B = B;
    a.ldb = ldb;
    a.C = C;
    a.ldc = ldc;
    a.k_slices = 1;
    a.slice_stride = 0;
    return a;
}

// Split-K plan: problems with few 64 x 64 output tiles and a long K are cut into K slices so that about 1024
// workgroups stream the operands.  A slice keeps at least 256 k when the tiles alone leave half the compute
// units idle, 1024 k when they would fill them once or twice; at most 64 slices, partial products within
// 16 MiB.  Depends on the shape only, so the order of summation, and with it the result, is the same on every
// call.  k_tile = 16 for fp32, 64 for bf16.  1 = do not split.
int splitk_slices(int64_t M, int64_t N, int64_t K, int k_tile)
{
    const int64_t tiles = ceil_div(M, 64) * ceil_div(N, 64), nk = ceil_div(K, k_tile);
    if (M == 0 || N == 0 || tiles > 512) return 1;
    int64_t s = 1024 / tiles;
    const int64_t longest = nk / ((tiles <= 128 ? 256 : 1024) / k_tile);
    if (s > longest) s = longest;
    if (s > 64) s = 64;
    const int64_t cap = ((int64_t)16 << 20) / (M * N * 4);
    if (s > cap) s = cap;
    return s < 2 ? 1 : (int)s;
}

}  // namespace

namespace fsrgemm {

hipError_t ensure_dynamic_lds(const void *kernel, int bytes, std::atomic<uint64_t> &done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < 64;
    const uint64_t bit = tracked ? (uint64_t)1 << dev : 0;
    if (tracked && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && tracked) done.fetch_or(bit, std::memory_order_release);
    return e;
}

}  // namespace fsrgemm

extern "C" {

int gemm_f32(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb, float *C,
             int64_t ldc, void *stream)
{
    return gemm_f32_ex(0, 0, M, N, K, A, lda, B, ldb, C, ldc, stream);
}

int gemm_f32_ex(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                int64_t ldb, float *C, int64_t ldc, void *stream)
{
    int rc = check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc);
    if (rc != FSRGEMM_OK) return rc;
    Plan p;
    rc = plan_f32(M, N, K, A, lda, B, ldb, &p);
    if (rc != FSRGEMM_OK) return rc;
    if (M == 0 || N == 0) return FSRGEMM_OK;
    rc = device_ok();
    if (rc != FSRGEMM_OK) return rc;
    const hipError_t e = launch_f32(p.cfg, p.mode, transA ? kMnContig : kKContig, transB ? kKContig : kMnContig,
                                    pack(M, N, K, A, lda, B, ldb, C, ldc), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FSRGEMM_OK : FSRGEMM_ERR_LAUNCH;
}

int gemm_bf16(int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
              float *C, int64_t ldc, void *stream)
{
    return gemm_bf16_ex(0, 1, M, N, K, A, lda, B, ldb, C, ldc, stream);
}

int gemm_bf16_ex(int transA, int transB, int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda,
                 const uint16_t *B, int64_t ldb, float *C, int64_t ldc, void *stream)
{
    int rc = check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc);
    if (rc != FSRGEMM_OK) return rc;
    const int a_lay = transA ? kMnContig : kKContig, b_lay = transB ? kKContig : kMnContig;
    Plan p;
    rc = plan_bf16(a_lay, b_lay, M, N, K, A, lda, B, ldb, &p);
    if (rc != FSRGEMM_OK) return rc;
    if (M == 0 || N == 0) return FSRGEMM_OK;
    rc = device_ok();
    if (rc != FSRGEMM_OK) return rc;
    const hipError_t e = launch_bf16(p.cfg, p.mode, a_lay, b_lay, pack(M, N, K, A, lda, B, ldb, C, ldc),
                                     static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FSRGEMM_OK : FSRGEMM_ERR_LAUNCH;
}

int64_t gemm_f32_workspace_bytes(int transA, int transB, int64_t M, int64_t N, int64_t K)
{
    (void)transA;
    (void)transB;
    if (M < 0 || N < 0 || K < 0 || M >= ((int64_t)1 << 31) || N >= ((int64_t)1 << 31) || K >= ((int64_t)1 << 31)) return 0;
    const int slices = splitk_slices(M, N, K, 16);
    return slices > 1 ? (int64_t)slices * M * N * 4 : 0;
}

int gemm_f32_ws(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                int64_t ldb, float *C, int64_t ldc, void *workspace, int64_t workspace_bytes, void *stream)
{
    int rc = check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc);
    if (rc != FSRGEMM_OK) return rc;
    if (workspace_bytes < 0 || (workspace_bytes > 0 && workspace == nullptr)) return FSRGEMM_ERR_INVALID_ARG;
    const int slices = splitk_slices(M, N, K, 16);
    const int64_t need = (int64_t)slices * M * N * 4;
    if (slices < 2 || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 3u))
        return gemm_f32_ex(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, stream);
    Plan p;
    rc = plan_f32(M, N, K, A, lda, B, ldb, &p);
    if (rc != FSRGEMM_OK) return rc;
    rc = device_ok();
    if (rc != FSRGEMM_OK) return rc;
    float *ws = static_cast<float *>(workspace);
    GemmArgs a = pack(M, N, K, A, lda, B, ldb, ws, N);
    a.k_slices = slices;
    a.slice_stride = M * N;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = launch_f32(p.cfg, p.mode, transA ? kMnContig : kKContig, transB ? kKContig : kMnContig, a, s);
    if (e == hipSuccess) e = launch_splitk_reduce(ws, slices, M * N, C, (int)M, (int)N, ldc, s);
    return e == hipSuccess ? FSRGEMM_OK : FSRGEMM_ERR_LAUNCH;
}

int64_t gemm_bf16_workspace_bytes(int transA, int transB, int64_t M, int64_t N, int64_t K)
{
    (void)transA;
    (void)transB;
    if (M < 0 || N < 0 || K < 0 || M >= ((int64_t)1 << 31) || N >= ((int64_t)1 << 31) || K >= ((int64_t)1 << 31)) return 0;
    const int slices = splitk_slices(M, N, K, 64);
    return slices > 1 ? (int64_t)slices * M * N * 4 : 0;
}

int gemm_bf16_ws(int transA, int transB, int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda,
                 const uint16_t *B, int64_t ldb, float *C, int64_t ldc, void *workspace, int64_t workspace_bytes,
                 void *stream)
{
    int rc = check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc);
    if (rc != FSRGEMM_OK) return rc;
    if (workspace_bytes < 0 || (workspace_bytes > 0 && workspace == nullptr)) return FSRGEMM_ERR_INVALID_ARG;
    const int slices = splitk_slices(M, N, K, 64);
    const int64_t need = (int64_t)slices * M * N * 4;
    if (slices < 2 || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 3u))
        return gemm_bf16_ex(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, stream);
    const int a_lay = transA ? kMnContig : kKContig, b_lay = transB ? kKContig : kMnContig;
    Plan p;
    rc = plan_bf16(a_lay, b_lay, M, N, K, A, lda, B, ldb, &p);
    if (rc != FSRGEMM_OK) return rc;
    if (p.cfg == kBf16_Main) return FSRGEMM_ERR_LAUNCH;      // cannot happen: a split problem has at most 512 small tiles
    rc = device_ok();
    if (rc != FSRGEMM_OK) return rc;
    float *ws = static_cast<float *>(workspace);
    GemmArgs a = pack(M, N, K, A, lda, B, ldb, ws, N);
    a.k_slices = slices;
    a.slice_stride = M * N;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = launch_bf16(p.cfg, p.mode, a_lay, b_lay, a, s);
    if (e == hipSuccess) e = launch_splitk_reduce(ws, slices, M * N, C, (int)M, (int)N, ldc, s);
    return e == hipSuccess ? FSRGEMM_OK : FSRGEMM_ERR_LAUNCH;
}

const char *fsrgemm_kernel_for_f32(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                                   int64_t ldb, const float *C, int64_t ldc)
{
    return fsrgemm_kernel_for_f32_ex(0, 0, M, N, K, A, lda, B, ldb, C, ldc);
}

const char *fsrgemm_kernel_for_f32_ex(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A,
                                      int64_t lda, const float *B, int64_t ldb, const float *C, int64_t ldc)
{
    Plan p;
    if (check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc) != FSRGEMM_OK) return nullptr;
    if (plan_f32(M, N, K, A, lda, B, ldb, &p) != FSRGEMM_OK) return nullptr;
    return f32_kernel_name(p.cfg, p.mode, transA ? kMnContig : kKContig, transB ? kKContig : kMnContig);
}

const char *fsrgemm_kernel_for_bf16(int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda,
                                    const uint16_t *B, int64_t ldb, const float *C, int64_t ldc)
{
    return fsrgemm_kernel_for_bf16_ex(0, 1, M, N, K, A, lda, B, ldb, C, ldc);
}

const char *fsrgemm_kernel_for_bf16_ex(int transA, int transB, int64_t M, int64_t N, int64_t K, const uint16_t *A,
                                       int64_t lda, const uint16_t *B, int64_t ldb, const float *C, int64_t ldc)
{
    Plan p;
    if (check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc) != FSRGEMM_OK) return nullptr;
    const int a_lay = transA ? kMnContig : kKContig, b_lay = transB ? kKContig : kMnContig;
    if (plan_bf16(a_lay, b_lay, M, N, K, A, lda, B, ldb, &p) != FSRGEMM_OK) return nullptr;
    return bf16_kernel_name(p.cfg, p.mode, a_lay, b_lay);
}

static bool transpose_args_ok(int64_t rows, int64_t cols, const float *A, int64_t lda, const float *T, int64_t ldt)
{
    const int64_t lim = (int64_t)1 << 31;
    if (rows < 0 || cols < 0 || rows >= lim || cols >= lim || lda < cols || ldt < rows) return false;
    if (rows == 0 || cols == 0) return true;
    return A != nullptr && T != nullptr && ceil_div(rows, 64) * ceil_div(cols, 64) < lim;
}

const char *fsrgemm_kernel_for_transpose_f32(int64_t rows, int64_t cols, const float *A, int64_t lda, const float *T, int64_t ldt)
{
    if (!transpose_args_ok(rows, cols, A, lda, T, ldt)) return nullptr;
    return rows == 0 || cols == 0 ? "none" : transpose_kernel_name((int)rows, (int)cols);
}

int transpose_f32(int64_t rows, int64_t cols, const float *A, int64_t lda, float *T, int64_t ldt, void *stream)
{
    if (!transpose_args_ok(rows, cols, A, lda, T, ldt)) return FSRGEMM_ERR_INVALID_ARG;
    if (rows == 0 || cols == 0) return FSRGEMM_OK;
    const int rc = device_ok();
    if (rc != FSRGEMM_OK) return rc;
    const hipError_t e = launch_transpose_f32(A, lda, T, ldt, (int)rows, (int)cols, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FSRGEMM_OK : FSRGEMM_ERR_LAUNCH;
}

const char *fsrgemm_status_string(int status)
{
    switch (status) {
    case FSRGEMM_OK: return "ok";
    case FSRGEMM_ERR_INVALID_ARG: return "invalid argument";
    case FSRGEMM_ERR_LAUNCH: return "kernel launch failed";
    case FSRGEMM_ERR_UNSUPPORTED_DEVICE: return "current device is not gfx950";
    default: return "unknown status";
    }
}

int fsrgemm_version(void) { return 100; }

}  // extern "C"
