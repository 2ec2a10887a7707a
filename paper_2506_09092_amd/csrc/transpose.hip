// fp32 matrix transposition for gfx950: T[cols x rows] with T[j][i] = A[i][j], both row-major (the paper's
// Task 8; its kernel analysis, Section 4.2.2, names what makes this operation fast: both the reads and the
// writes coalesced, the exchange done in on-chip memory without bank conflicts).
//
// The operation moves every element once in and once out, so HBM bandwidth bounds it.  One workgroup of 256
// lanes moves a TR x TC tile (64 x 128; 64 x 64 for matrices with fewer than 128 columns; 32 x 64 for small ones) through LDS:
// TC / 4 lanes read a contiguous piece of an input row (16 bytes each), the values are written to LDS
// transposed, and after a barrier TR / 4 lanes write a contiguous piece of an output row.  The LDS tile has
// rows of TR + 1 words: both the transposed writes and the row reads hit 64 different banks.
//
// Tiles are walked diagonally (tile column = (id % columns + tile row) % columns): workgroups that run at
// the same time then write to output rows that are spread over the whole matrix instead of to one band of
// them, which spreads the traffic over the memory channels (measured: +12 % at 64 x 64 tiles).
//
// A matrix that is not a whole number of tiles has its last tile row and column shifted back so that they end
// with the matrix (tile_origin): the overlap is moved twice, to the same place with the same bits, and no
// access of a full tile can leave the matrix.  Only matrices with fewer than 64 rows or columns take the
// element-wise, bounds-checked path.  Global accesses are written as 16-byte copies: the compiler emits
// 128-bit loads and stores, which this target allows at any address that is aligned for a float.
#include "launchers.hpp"

namespace fsrgemm {
namespace {

constexpr int kThreads = 256;

// CHECKED: the matrix is narrower than the tile in one direction; element by element, every access checked
template <int TR, int TC, bool CHECKED>
__global__ __launch_bounds__(kThreads) void transpose_f32_kernel(const float *__restrict__ A, int64_t lda, float *__restrict__ T,
                                                                 int64_t ldt, int rows, int cols, int tiles_r, int tiles_c)
{
    __shared__ float tile[TC][TR + 1];      // tile[j][i] = A[r0 + i][c0 + j]
    const int tr = (int)blockIdx.x / tiles_c;
    const int tc = ((int)blockIdx.x - tr * tiles_c + tr) % tiles_c;
    const int r0 = tile_origin(tr, TR, rows), c0 = tile_origin(tc, TC, cols);
    const int tid = threadIdx.x;
    (void)tiles_r;

    if constexpr (!CHECKED) {
        constexpr int VX = TC / 4, PY = kThreads / VX, NP = TR / PY;      // vectors per input row piece, rows per pass, passes
        const int x = tid % VX, y = tid / VX;
        f32x4 v[NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) __builtin_memcpy(&v[p], A + (int64_t)(r0 + y + PY * p) * lda + c0 + 4 * x, sizeof(f32x4));
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int e = 0; e < 4; ++e) tile[4 * x + e][y + PY * p] = v[p][e];
        __syncthreads();
        constexpr int WX = TR / 4, QY = kThreads / WX, NQ = TC / QY;      // the same for the output rows
        const int wx = tid % WX, wy = tid / WX;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            f32x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = tile[wy + QY * q][4 * wx + e];
            __builtin_memcpy(T + (int64_t)(c0 + wy + QY * q) * ldt + r0 + 4 * wx, &w, sizeof(f32x4));
        }
    } else {
        for (int idx = tid; idx < TR * TC; idx += kThreads) {
            const int i = idx / TC, j = idx % TC;
            if (r0 + i < rows && c0 + j < cols) tile[j][i] = A[(int64_t)(r0 + i) * lda + c0 + j];
        }
        __syncthreads();
        for (int idx = tid; idx < TR * TC; idx += kThreads) {
            const int j = idx / TR, i = idx % TR;
            if (r0 + i < rows && c0 + j < cols) T[(int64_t)(c0 + j) * ldt + r0 + i] = tile[j][i];
        }
    }
}

template <int TR, int TC, bool CHECKED>
hipError_t launch(const float *A, int64_t lda, float *T, int64_t ldt, int rows, int cols, hipStream_t s)
{
    const int tiles_r = (rows + TR - 1) / TR, tiles_c = (cols + TC - 1) / TC;
    hipLaunchKernelGGL((transpose_f32_kernel<TR, TC, CHECKED>), dim3((unsigned)(tiles_r * tiles_c)), dim3(kThreads), 0, s, A, lda, T,
                       ldt, rows, cols, tiles_r, tiles_c);
    return hipGetLastError();
}

}  // namespace

// A matrix that gives the 64 x 128 tile no more than two workgroups per compute unit is moved in 32 x 64 tiles: such a
// launch is a few microseconds of latency, not of bandwidth, and four times the workgroups hide more of it (kernel
// time 1024^2 3.4 -> 3.0 us, 2048^2 6.5 -> 5.3; level at 4096^2, 8 % slower at 8192^2 and beyond).
static bool small_matrix(int rows, int cols) { return (int64_t)((rows + 63) / 64) * ((cols + 127) / 128) <= 512; }

// <tile rows, tile columns, checked>: as a profiler trace prints the kernel
const char *transpose_kernel_name(int rows, int cols)
{
    if (rows < 64 || cols < 64) return "transpose_f32_kernel<64, 64, true>";
    if (small_matrix(rows, cols)) return "transpose_f32_kernel<32, 64, false>";
    return cols >= 128 ? "transpose_f32_kernel<64, 128, false>" : "transpose_f32_kernel<64, 64, false>";
}

// rows, cols >= 1; the number of 64 x 64 tiles must fit a grid (checked by the caller)
hipError_t launch_transpose_f32(const float *A, int64_t lda, float *T, int64_t ldt, int rows, int cols, hipStream_t s)
{
    if (rows < 64 || cols < 64) return launch<64, 64, true>(A, lda, T, ldt, rows, cols, s);
    if (small_matrix(rows, cols)) return launch<32, 64, false>(A, lda, T, ldt, rows, cols, s);
    if (cols >= 128) return launch<64, 128, false>(A, lda, T, ldt, rows, cols, s);
    return launch<64, 64, false>(A, lda, T, ldt, rows, cols, s);
}

}  // namespace fsrgemm
