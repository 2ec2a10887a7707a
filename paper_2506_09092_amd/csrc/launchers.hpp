// Host-side interface between the C ABI (api.hip) and the kernel files: configuration numbers, kernel names as
// a profiler prints them, and one launcher per kernel family.
#pragma once
#include <atomic>

#include "common.hpp"

namespace fsrgemm {

// Raises a kernel's dynamic-LDS limit once per device (the attribute belongs to the device's copy of the
// kernel).  `done` is the caller's per-kernel bitmap of devices already configured; safe to call concurrently.
hipError_t ensure_dynamic_lds(const void *kernel, int bytes, std::atomic<uint64_t> &done);

// fp32 tile configurations (gemm_f32.hip), each available in the three load modes and the four layout pairs
enum F32Config { kF32_256x128 = 0, kF32_128x128 = 1, kF32_64x64 = 2, kF32ConfigCount };
// the unchecked load mode addresses a lane's vectors with 32-bit byte offsets: leading dimensions below this
constexpr int64_t kF32MaxLdUnchecked = (int64_t)1 << 24;
// Names are substrings of the kernel symbols as a profiler trace prints them.
const char *f32_kernel_name(int cfg, int mode, int a_lay, int b_lay);
hipError_t launch_f32(int cfg, int mode, int a_lay, int b_lay, const GemmArgs &a, hipStream_t s);
// second half of a split-K product: C = sum over slices, in slice order
const char *splitk_reduce_kernel_name();
hipError_t launch_splitk_reduce(const float *ws, int slices, int64_t slice_stride, float *C, int M, int N, int64_t ldc,
                                hipStream_t s);

// bf16 configurations: the direct-to-LDS 256x256 kernel for large aligned problems (gemm_bf16_main.hip, the
// four layout pairs) and three tile sizes of the general kernel (gemm_bf16.hip), each in the three load
// modes and the four layout pairs
enum Bf16Config { kBf16_Main = 0, kBf16_256x256 = 1, kBf16_128x128 = 2, kBf16_64x64 = 3, kBf16ConfigCount };
const char *bf16_kernel_name(int cfg, int mode, int a_lay, int b_lay);
hipError_t launch_bf16(int cfg, int mode, int a_lay, int b_lay, const GemmArgs &a, hipStream_t s);
// the direct-to-LDS kernel's tile shapes: 256 x 256 (candidate kBf16_Main), then 192 x 256, 128 x 256, 256 x 192,
// 192 x 192, 256 x 128, 128 x 128 (candidates kBf16_MainMore ..., after the vector kernels); no K slices
constexpr int kBf16MainShapes = 7;
int bf16_main_tile_m(int shape);
int bf16_main_tile_n(int shape);
bool bf16_main_fits(int shape, int a_lay, int b_lay, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb);
const char *bf16_main_kernel_name(int shape, int a_lay, int b_lay);
bool bf16_main_slices_fit(int64_t K, int slices);      // K slices of whole K-tiles, the last with at least one
hipError_t launch_bf16_main(int shape, int a_lay, int b_lay, const GemmArgs &a, hipStream_t s);

// fp32 products with M == 1 or N == 1 (gemv_f32.hip): y[i * incy] = sum over k of mat(i, k) * x[k * incx] for
// i < len, with mat(i, k) at mat[i * ld + k] (kVecRows) or mat[k * ld + i] (kVecCols).  With k_slices > 1 slice s
// writes its partial y behind y + s * slice_stride.  xvec is filled in by the launcher.
enum VecPattern { kVecRows = 0, kVecCols = 1 };
constexpr int kF32_Vector = kF32ConfigCount;        // the candidate number of these kernels, after the tile configurations
struct VecArgs {
    const float *mat;
    int64_t ld;
    const float *x;
    int64_t incx;
    float *y;
    int64_t incy;
    int len, K;
    int k_slices;
    int64_t slice_stride;
    bool xvec;
    int nvec;               // vectors x_r = x + r * ldx, y_r = y + r * ldy, r < nvec <= kMaxFewVectorsF32
    int64_t ldx, ldy;
};
constexpr int kMaxFewVectors = 8;           // bf16, lane arithmetic
constexpr int kMaxFewVectorsF32 = 16;
const char *gemv_kernel_name(int pattern, bool vec, int nvec = 1);
bool gemv_takes_vectors(const VecArgs &a);
bool gemv_takes_few(int pattern, const VecArgs &a);     // whether a.nvec > 1 vectors can go through these kernels
hipError_t launch_gemv_f32(int pattern, VecArgs a, hipStream_t s);

// the same for bf16 operands (gemv_bf16.hip); y is fp32
constexpr int kBf16_Vector = kBf16ConfigCount;      // the candidate number of these kernels, after the tile configurations
constexpr int kBf16_MainMore = kBf16_Vector + 1;    // candidate number of the direct-to-LDS kernel's second shape
// shape of the direct-to-LDS kernel a bf16 candidate number stands for, -1 if none
inline int bf16_main_shape(int cfg)
{
    return cfg == kBf16_Main ? 0 : cfg >= kBf16_MainMore && cfg < kBf16_MainMore + kBf16MainShapes - 1 ? cfg - kBf16_MainMore + 1 : -1;
}
inline int bf16_main_candidate(int shape) { return shape == 0 ? (int)kBf16_Main : kBf16_MainMore + shape - 1; }
struct VecArgs16 {
    const uint16_t *mat;
    int64_t ld;
    const uint16_t *x;
    int64_t incx;
    float *y;
    int64_t incy;
    int len, K;
    int k_slices;
    int64_t slice_stride;
    bool xvec;
    int nvec;               // vectors x_r = x + r * ldx, y_r = y + r * ldy, r < nvec <= kMaxFewVectors (kMaxMfmaVectors)
    int64_t ldx, ldy;
};
constexpr int kMaxMfmaVectors = 16;
constexpr int kMfmaDirectVectors = 8;       // up to here the matrix-core kernel reads the vectors' fragments straight from global memory
const char *gemv_bf16_kernel_name(int pattern, bool vec, int nvec = 1, bool mfma = false);
bool gemv_bf16_takes_vectors(const VecArgs16 &a);
bool gemv_bf16_takes_few(int pattern, const VecArgs16 &a);      // whether a.nvec > 1 vectors can go through these kernels
bool gemv_bf16_takes_mfma(int pattern, const VecArgs16 &a);     // whether the matrix-core kernel takes them (then it is the one launched)
hipError_t launch_gemv_bf16(int pattern, VecArgs16 a, hipStream_t s);

// fp32 products with M, N <= 16 and a long K, both operands stored with k as the row index (gemm_f32_skinny.hip):
// element (i, k) of A at A[k * lda + i], element (k, j) of B at B[k * ldb + j]; K is cut into `parts` pieces whose
// partial results go to partial[part][M][N] and are then added into C.
constexpr int kF32_Skinny = kF32_Vector + 1;        // candidate number, after the vector kernels
constexpr int kSkinnyMaxParts = 256;
struct SkinnyArgs {
    const float *A;
    int64_t lda;
    const float *B;
    int64_t ldb;
    int M, N, K;
    int parts;
    float *partial;
};
bool skinny_fits(int64_t M, int64_t N);
bool skinny_offsets_fit(const SkinnyArgs &a);
const char *skinny_kernel_name(int M, int N, const float *A, int64_t lda, const float *B, int64_t ldb);
hipError_t launch_skinny_f32(const SkinnyArgs &a, float *C, int64_t ldc, hipStream_t s);

// fp32 direct-to-LDS kernel for aligned problems (gemm_f32_main.hip), no K slices: twelve tile shapes -- 256 x 256,
// 192 x 256, 128 x 256, 256 x 128, 192 x 128, 128 x 128, 256 x 192, 192 x 192, 128 x 192, 64 x 64, 128 x 64, 64 x 128 -- in
// the four layout pairs
constexpr int kF32_Main = kF32_Skinny + 1;          // candidate number of the first shape, after the small-result kernel
constexpr int kF32MainShapes = 12;
int f32_main_tile_m(int shape);
int f32_main_tile_n(int shape);
bool f32_main_fits(int shape, int a_lay, int b_lay, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb);
const char *f32_main_kernel_name(int shape, int a_lay, int b_lay);
bool f32_main_slices_fit(int64_t K, int slices);       // K slices of whole K-tiles, the last with at least one
hipError_t launch_f32_main(int shape, int a_lay, int b_lay, const GemmArgs &a, hipStream_t s);

// register-only MFMA loops (mfma_ceiling.hip): kind 0 = the fp32 kernels' instruction, 1 = the bf16 kernels'
const char *mfma_ceiling_kernel_name(int kind);
double mfma_ceiling_flop(int kind, int passes, int workgroups);
hipError_t launch_mfma_ceiling(int kind, int passes, const void *operands, float *sink, int workgroups, hipStream_t s);

// fp32 transposition (transpose.hip)
const char *transpose_kernel_name(int rows, int cols);
hipError_t launch_transpose_f32(const float *A, int64_t lda, float *T, int64_t ldt, int rows, int cols, hipStream_t s);

}  // namespace fsrgemm
