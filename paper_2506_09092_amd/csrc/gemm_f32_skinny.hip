// fp32 products with a small output and a long K: C[M x N] = A . B with M, N <= 16 and K in the thousands to
// millions -- the normal equations X^T X and X^T y of the paper's Task 20 (ordinary least squares, 2^14 .. 2^22
// samples of 10 features) are the case in point.  Every operand element is used M or N times at most, so the
// product is bound by streaming A and B from HBM once: 4 (M + N) K bytes; the matrix cores would spend their time
// on padding (a 32 x 32 block for a 10 x 10 result), so the sums are plain vector FMAs.
//
// The K range is cut into `parts` pieces, one per workgroup.  Inside a workgroup every lane walks its piece in
// steps of 256, keeps the whole MB x NB result (M, N rounded up to multiples of 4) in registers and adds one outer
// product a_k b_k^T per step.  The 256 private results are then added in a fixed order through LDS -- lane by lane
// inside each wavefront, then the four wavefronts -- and the workgroup's partial result goes to its own M x N
// block of the workspace.  A second kernel, one wavefront per output element, adds the partial results in a fixed order
// too, so the product repeats bit for bit.
//
// Both operands are taken in the storage of that task: tall matrices with k as the row index (A stored K x M,
// B stored K x N, i.e. a transposed A and a row-major B).  Along k the lanes of a wavefront read consecutive rows,
// 64 rows being one contiguous run of memory for a tightly packed operand.  Other storage orders of such shapes
// stay with the split tile kernels.
#include <stdio.h>

#include "launchers.hpp"

namespace fsrgemm {

namespace {

constexpr int kThreads = 256;

// (an even M only: the pair that holds the last element of an odd M would reach one element into the row's padding)
bool skinny_reads_pairs(const SkinnyArgs &a) { return (reinterpret_cast<uintptr_t>(a.A) & 7u) == 0 && a.lda % 2 == 0 && a.M % 2 == 0; }
bool skinny_is_gram(const SkinnyArgs &a) { return a.A == a.B && a.M == a.N && a.lda == a.ldb; }

// APAIR: A's rows start 8-byte aligned (base and leading dimension even) and M is even, so a row is read as pairs.
// GRAM: X^T X -- A and B are the same matrix, so one set of loads serves both, and the result is symmetric, so only
// j >= i is summed and the rest copied over at the end (the same products in the same order: the copy has the
// bits the sum would have had).
template <int MB, int NB, bool APAIR, bool GRAM>
__global__ __launch_bounds__(kThreads) void gemm_f32_skinny_kernel(SkinnyArgs g)
{
    constexpr int V = MB * NB;                      // private sums per lane
    constexpr int CH = V < 36 ? V : 36;             // of which this many go through LDS at a time
    __shared__ float red[4 * CH][65];               // [wavefront, value][lane], rows padded against bank conflicts
    __shared__ float wsum[4][V];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t per = ((int64_t)g.K + g.parts - 1) / g.parts;
    const int64_t k0 = min((int64_t)blockIdx.x * per, (int64_t)g.K), k1 = min(k0 + per, (int64_t)g.K);
    const int len = (int)(k1 - k0);
    // Addresses are a uniform base (the piece's first row) plus a 32-bit lane offset (the row) plus a constant (the
    // column): the launcher has checked that the offsets inside a piece stay below 2^29 elements.
    const float *__restrict__ A = g.A + k0 * g.lda;
    const float *__restrict__ B = g.B + k0 * g.ldb;
    const uint32_t lda = (uint32_t)g.lda, ldb = (uint32_t)g.ldb;
    float acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = 0.f;

    // Row kk < len of the piece.  The padding of the register block reads the row's last valid element and is set
    // to zero afterwards, so no load sits behind a branch and the loads of a batch are issued back to back.
    auto row = [&](int kk, float (&a)[MB], float (&b)[NB]) {
        const float *__restrict__ ar = A + (uint32_t)kk * lda;
        const float *__restrict__ br = B + (uint32_t)kk * ldb;
        if constexpr (APAIR) {
            typedef float f32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int i = 0; i < MB; i += 2) {
                const f32x2 v = *reinterpret_cast<const f32x2 *>(ar + min(i, g.M - 2));
                a[i] = i < g.M ? v[0] : 0.f;
                a[i + 1] = i + 1 < g.M ? v[1] : 0.f;
            }
        } else {
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                const float v = ar[min(i, g.M - 1)];
                a[i] = i < g.M ? v : 0.f;
            }
        }
        if constexpr (!GRAM) {
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const float v = br[min(j, g.N - 1)];
                b[j] = j < g.N ? v : 0.f;
            }
        }
    };
    // Whole batches of U rows per lane: all loads of a batch are issued, then its rows are added to the private
    // result.  The rows behind the last whole batch follow one at a time.
    constexpr int U = V <= 64 ? 8 : 4;
    constexpr int kBatch = U * kThreads;
    auto add_row = [&](const float (&ar)[MB], const float (&br)[NB]) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = GRAM ? i : 0; j < NB; ++j) acc[i][j] = __builtin_fmaf(ar[i], GRAM ? ar[j] : br[j], acc[i][j]);
    };
    int kk = tid;
    for (; kk + (U - 1) * kThreads < len; kk += kBatch) {
        float a[U][MB], b[U][NB];
#pragma unroll
        for (int u = 0; u < U; ++u) row(kk + u * kThreads, a[u], b[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) add_row(a[u], b[u]);
    }
    for (; kk < len; kk += kThreads) {
        float ar[MB], br[NB];
        row(kk, ar, br);
        add_row(ar, br);
    }

    if constexpr (GRAM) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < i; ++j) acc[i][j] = acc[j][i];
    }

    // 256 private results -> 1, in a fixed order: CH values at a time every lane parks its sums in LDS, then one
    // lane per (wavefront, value) adds the 64 of them in lane order; at the end the four wavefronts in order
#pragma unroll
    for (int c = 0; c < V; c += CH) {
#pragma unroll
        for (int v = 0; v < CH; ++v)
            if (c + v < V) red[wave * CH + v][lane] = acc[(c + v) / NB][(c + v) % NB];
        __syncthreads();
        if (tid < 4 * CH && c + tid % CH < V) {
            float s = red[tid][0];
            for (int l = 1; l < 64; ++l) s += red[tid][l];
            wsum[tid / CH][c + tid % CH] = s;
        }
        __syncthreads();
    }
    if (tid < V) {
        const int i = tid / NB, j = tid % NB;
        if (i < g.M && j < g.N)
            g.partial[(int64_t)blockIdx.x * g.M * g.N + i * g.N + j] = ((wsum[0][tid] + wsum[1][tid]) + wsum[2][tid]) + wsum[3][tid];
    }
}

// C[i][j] = sum of the partial results, one wavefront per output element: lane l adds partials l, l + 64, ... in
// that order, then the butterfly
__global__ __launch_bounds__(64) void skinny_reduce_kernel(const float *__restrict__ partial, int parts, int M, int N,
                                                           float *__restrict__ C, int64_t ldc)
{
    const int e = blockIdx.x, lane = threadIdx.x;
    float s = 0.f;
    for (int p = lane; p < parts; p += 64) s += partial[(int64_t)p * M * N + e];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d, 64);
    if (lane == 0) C[(int64_t)(e / N) * ldc + e % N] = s;
}

template <int MB, int NB>
hipError_t launch(const SkinnyArgs &a, hipStream_t s)
{
    const dim3 grid((unsigned)a.parts), block(kThreads);
    if constexpr (MB == NB) {
        if (skinny_is_gram(a)) {
            if (skinny_reads_pairs(a)) hipLaunchKernelGGL((gemm_f32_skinny_kernel<MB, NB, true, true>), grid, block, 0, s, a);
            else hipLaunchKernelGGL((gemm_f32_skinny_kernel<MB, NB, false, true>), grid, block, 0, s, a);
            return hipGetLastError();
        }
    }
    if (skinny_reads_pairs(a)) hipLaunchKernelGGL((gemm_f32_skinny_kernel<MB, NB, true, false>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((gemm_f32_skinny_kernel<MB, NB, false, false>), grid, block, 0, s, a);
    return hipGetLastError();
}

template <int MB>
hipError_t launch_m(int nb, const SkinnyArgs &a, hipStream_t s)
{
    switch (nb) {
    case 4: return launch<MB, 4>(a, s);
    case 8: return launch<MB, 8>(a, s);
    case 12:
        if constexpr (MB <= 12) return launch<MB, 12>(a, s);
        break;
    case 16:
        if constexpr (MB <= 8) return launch<MB, 16>(a, s);
        break;
    }
    return hipErrorInvalidValue;
}

int round4(int x) { return (x + 3) / 4 * 4; }

}  // namespace

// register blocks exist for M, N rounded up to multiples of 4 with at most 144 accumulators
bool skinny_fits(int64_t M, int64_t N)
{
    return M >= 1 && N >= 1 && M <= 16 && N <= 16 && round4((int)M) * round4((int)N) <= 144;
}

// <MB, NB, A read as pairs, X^T X> as a profiler trace prints the kernel
const char *skinny_kernel_name(int M, int N, const float *A, int64_t lda, const float *B, int64_t ldb)
{
    struct Names {
        char text[4][4][2][2][56];
        Names()
        {
            for (int i = 0; i < 4; ++i)
                for (int j = 0; j < 4; ++j)
                    for (int p = 0; p < 2; ++p)
                        for (int q = 0; q < 2; ++q)
                            snprintf(text[i][j][p][q], sizeof text[i][j][p][q], "gemm_f32_skinny_kernel<%d, %d, %s, %s>", 4 * i + 4,
                                     4 * j + 4, p ? "true" : "false", q ? "true" : "false");
        }
    };
    static const Names names;
    if (!skinny_fits(M, N)) return nullptr;
    SkinnyArgs a;
    a.A = A, a.lda = lda, a.B = B, a.ldb = ldb, a.M = M, a.N = N;
    return names.text[round4(M) / 4 - 1][round4(N) / 4 - 1][skinny_reads_pairs(a)][skinny_is_gram(a)];
}

// the lane offsets inside one piece of K are 32-bit: the farthest element of a piece must stay below 2^29
bool skinny_offsets_fit(const SkinnyArgs &a)
{
    const int64_t per = ((int64_t)a.K + a.parts - 1) / a.parts, lim = (int64_t)1 << 29;
    return per * a.lda < lim && per * a.ldb < lim;
}

// skinny_fits(M, N), skinny_offsets_fit(a), K >= 1, 1 <= parts <= 256; partial holds parts * M * N floats
hipError_t launch_skinny_f32(const SkinnyArgs &a, float *C, int64_t ldc, hipStream_t s)
{
    if (!skinny_fits(a.M, a.N) || !skinny_offsets_fit(a)) return hipErrorInvalidValue;
    hipError_t e;
    switch (round4(a.M)) {
    case 4: e = launch_m<4>(round4(a.N), a, s); break;
    case 8: e = launch_m<8>(round4(a.N), a, s); break;
    case 12: e = launch_m<12>(round4(a.N), a, s); break;
    default: e = launch_m<16>(round4(a.N), a, s); break;
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(skinny_reduce_kernel, dim3((unsigned)(a.M * a.N)), dim3(64), 0, s, a.partial, a.parts, a.M, a.N, C, ldc);
    return hipGetLastError();
}

}  // namespace fsrgemm
