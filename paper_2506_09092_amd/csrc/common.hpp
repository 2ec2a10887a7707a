// Shared device/host helpers for the gfx950 GEMM kernels: vector types, the
// workgroup-id -> output-tile mapping and the launcher declarations that the
// C ABI in api.hip dispatches to.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace fsrgemm {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;     // CDNA wavefront width
constexpr int kXcds = 8;      // MI355X: 8 accelerator dies, each with a private L2
constexpr int kGroupM = 8;    // tile rows walked together inside one die's share

// Workgroups are handed to the 8 dies round-robin (id % 8).  Re-number them so
// that each die owns one contiguous run of the tile sequence, then walk that
// sequence in column-major order inside bands of kGroupM tile rows.  A die's
// resident workgroups then share a few A row-panels and B column-panels in its
// own L2 instead of every die streaming every panel.
__device__ __forceinline__ void tile_coords(int pid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int total = tiles_m * tiles_n;
    const int per = total / kXcds, rem = total % kXcds;
    const int xcd = pid % kXcds, loc = pid / kXcds;
    const int lin = xcd < rem ? xcd * (per + 1) + loc : rem * (per + 1) + (xcd - rem) * per + loc;
    const int width = kGroupM * tiles_n;
    const int band = lin / width;
    const int first_m = band * kGroupM;
    const int rows = min(tiles_m - first_m, kGroupM);
    const int in_band = lin - band * width;
    tm = first_m + in_band % rows;
    tn = in_band / rows;
}

// First row (or column) of output tile `tile` when tiles are `size` wide and the matrix has `extent` rows.
// The last tile of a matrix that is not a whole number of tiles is shifted back so that it ends with the
// matrix: it then overlaps its neighbour, both compute the overlap with the same operands in the same order
// and store the same bits, and no load or store of a full tile can leave the matrix.  Matrices narrower than
// one tile keep their single tile at 0 and need checked loads and stores.
__device__ __forceinline__ int tile_origin(int tile, int size, int extent)
{
    return extent >= size ? min(tile * size, extent - size) : 0;
}

// Raises a kernel's dynamic-LDS limit once per device (the attribute belongs to the device's copy of the
// kernel).  `done` is the caller's per-kernel bitmap of devices already configured; safe to call concurrently.
hipError_t ensure_dynamic_lds(const void *kernel, int bytes, std::atomic<uint64_t> &done);

struct GemmArgs {
    int M, N, K;
    const void *A;
    int64_t lda;
    const void *B;
    int64_t ldb;
    float *C;
    int64_t ldc;
    // split-K (fp32 kernels and the general bf16 kernel): number of K slices (1 = none) and the distance in floats between the partial
    // products of consecutive slices behind C
    int k_slices;
    int64_t slice_stride;
};

// How global loads are issued.
//   kFast:    16-byte vectors, no bounds checks (aligned, tile-multiple shapes)
//   kVecPred: 16-byte vectors where a whole vector is in range, element-wise
//             zero-filled loads at the ragged edge (aligned bases and lds)
//   kScalar:  element-wise predicated loads (any alignment, any shape)
// Kernels are instantiated for these three; inside a kernel the whole K-tiles of a tile that lies inside the
// matrix are loaded without checks in every mode: as kFast, or, in a kScalar kernel, as
//   kUnalignedVec: 16-byte loads from addresses with only the element's alignment, no bounds checks (the
//             compiler picks the widest load the target allows for such an address)
enum LoadMode { kFast = 0, kVecPred = 1, kScalar = 2, kUnalignedVec = 3 };

// Which index of an operand tile is contiguous in memory: k (a row-major A, a transposed B) or the
// m / n index (a transposed A, a row-major B).
enum OperandLayout { kKContig = 0, kMnContig = 1 };

// fp32 tile configurations (gemm_f32.hip), each available in the three load modes and the four layout pairs
enum F32Config { kF32_256x128 = 0, kF32_128x128 = 1, kF32_64x64 = 2, kF32ConfigCount };
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
const char *bf16_main_kernel_name(int a_lay, int b_lay);
hipError_t launch_bf16_main(int a_lay, int b_lay, const GemmArgs &a, hipStream_t s);

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
};
const char *gemv_kernel_name(int pattern, bool vec);
bool gemv_takes_vectors(const VecArgs &a);
hipError_t launch_gemv_f32(int pattern, VecArgs a, hipStream_t s);

// fp32 transposition (transpose.hip)
const char *transpose_kernel_name(int rows, int cols);
hipError_t launch_transpose_f32(const float *A, int64_t lda, float *T, int64_t ldt, int rows, int cols, hipStream_t s);

}  // namespace fsrgemm
