// Shared device helpers and argument types of the gfx950 kernels: vector types, the
// workgroup-id -> output-tile mapping, the shifted edge tiles, load modes and operand layouts.
// What the C ABI in api.hip dispatches to is declared in launchers.hpp.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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

}  // namespace fsrgemm
