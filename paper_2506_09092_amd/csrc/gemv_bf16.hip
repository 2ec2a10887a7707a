// bf16 products in which M or N is 1 (a vector on one side), fp32 sums and output: the bf16 twin of gemv_f32.hip,
// the shape of a single-token step against a weight matrix.  The matrix streams from HBM exactly once, so
// bandwidth bounds the kernel: 2 (M K + K N) + 4 M N bytes.  Two access patterns cover the four storage cases:
//   rows:  the matrix is contiguous along the summation index, y[r] = sum_k Mat[r][k] x[k] (a row times a
//          column-major B -- what gemm_bf16 takes -- or a row-major A times a column).  One wavefront per row: its
//          lanes read 16-byte pieces (8 values) 1 KB apart, four in flight, multiply by the matching piece of x
//          (served from cache) and the 64 partial sums are added in a fixed butterfly.
//   cols:  the matrix is contiguous along the output index, y[j] = sum_k x[k] Mat[k][j].  One workgroup per 64
//          output columns (one 128-byte line of every matrix row): 8 lanes cover the line, 32 groups of lanes
//          take every 32nd row, eight rows in flight each, and the 32 partial sums per column are added in
//          group order through LDS.
// Values are widened to fp32 (exact), products and sums are fp32 FMAs.  With k_slices > 1 the K range is cut
// into slices that write partial results behind g.y (a workspace), added afterwards by the split-K reduction
// kernel.  All sums have a fixed order: results repeat bit for bit.
#include "launchers.hpp"

namespace fsrgemm {

namespace {

constexpr int kThreads = 256;

typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float widen(uint16_t h) { return __builtin_bit_cast(float, (uint32_t)h << 16); }
__device__ __forceinline__ u16x8 load8(const uint16_t *p) { return *reinterpret_cast<const u16x8 *>(p); }

// x[k .. k + 7], as one vector when x is contiguous and 16-byte aligned
__device__ __forceinline__ u16x8 load_x8(const uint16_t *x, int64_t incx, bool xvec, int k)
{
    if (xvec) return load8(x + k);
    u16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = x[(int64_t)(k + e) * incx];
    return v;
}

__device__ __forceinline__ float dot8(u16x8 a, u16x8 b, float acc)
{
#pragma unroll
    for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(widen(a[e]), widen(b[e]), acc);
    return acc;
}

// VEC: the matrix base is 16-byte aligned and ld a multiple of 8, so 16-byte loads of whole pieces are aligned
template <bool VEC>
__global__ __launch_bounds__(kThreads) void gemv_rows_bf16_kernel(VecArgs16 g)
{
    const int groups = (g.len + 3) / 4;                       // four rows per workgroup, one per wavefront
    const int slice = (int)blockIdx.x / groups;
    const int r = ((int)blockIdx.x - slice * groups) * 4 + ((int)threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (r >= g.len) return;
    // slices start at multiples of 8 so that vector loads stay aligned
    const int per = (((g.K + g.k_slices - 1) / g.k_slices) + 7) & ~7;
    const int k0 = min((int64_t)slice * per, (int64_t)g.K), k1 = min((int64_t)k0 + per, (int64_t)g.K);
    const uint16_t *__restrict__ row = g.mat + (int64_t)r * g.ld;
    const uint16_t *__restrict__ x = g.x;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    if constexpr (VEC) {
        int k = k0 + 8 * lane;
        for (; k + 1543 < k1; k += 2048) {
            u16x8 m[4], v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) m[u] = load8(row + k + 512 * u);
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = load_x8(x, g.incx, g.xvec, k + 512 * u);
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] = dot8(m[u], v[u], acc[u]);
        }
        for (; k + 7 < k1; k += 512) acc[0] = dot8(load8(row + k), load_x8(x, g.incx, g.xvec, k), acc[0]);
        const int kt = k0 + ((k1 - k0) & ~7) + lane;           // the up to seven elements behind the last whole piece
        if (lane < ((k1 - k0) & 7)) acc[1] = __builtin_fmaf(widen(row[kt]), widen(x[(int64_t)kt * g.incx]), acc[1]);
    } else {
        int k = k0 + lane;
        for (; k + 192 < k1; k += 256) {
            uint16_t m[4], v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) m[u] = row[k + 64 * u];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = x[(int64_t)(k + 64 * u) * g.incx];
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] = __builtin_fmaf(widen(m[u]), widen(v[u]), acc[u]);
        }
        for (; k < k1; k += 64) acc[0] = __builtin_fmaf(widen(row[k]), widen(x[(int64_t)k * g.incx]), acc[0]);
    }
    float s = (acc[0] + acc[1]) + (acc[2] + acc[3]);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d, 64);
    if (lane == 0) g.y[(int64_t)slice * g.slice_stride + (int64_t)r * g.incy] = s;
}

template <bool VEC>
__global__ __launch_bounds__(kThreads) void gemv_cols_bf16_kernel(VecArgs16 g)
{
    constexpr int CW = 64;                                    // output columns per workgroup: 128 bytes of a matrix row
    constexpr int LANES = VEC ? 8 : 64, PER = CW / LANES;     // lanes across the columns, columns per lane
    constexpr int KG = kThreads / LANES;                      // groups of lanes that share the rows among them
    constexpr int UNROLL = 8;
    __shared__ float red[KG][CW + 1];
    const int groups = (g.len + CW - 1) / CW;
    const int slice = (int)blockIdx.x / groups;
    const int j0 = ((int)blockIdx.x - slice * groups) * CW;
    const int tid = threadIdx.x, cl = tid % LANES, kg = tid / LANES;
    const int per = (g.K + g.k_slices - 1) / g.k_slices;
    const int k0 = min((int64_t)slice * per, (int64_t)g.K), k1 = min((int64_t)k0 + per, (int64_t)g.K);
    const int j = j0 + cl * PER;
    const uint16_t *__restrict__ col = g.mat + j;
    const uint16_t *__restrict__ x = g.x;
    float acc[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) acc[e] = 0.f;

    bool done = false;
    if constexpr (VEC) {
        if (j + 7 < g.len) {
            int k = k0 + kg;
            for (; k + (UNROLL - 1) * KG < k1; k += UNROLL * KG) {
                u16x8 m[UNROLL];
                float v[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) m[u] = load8(col + (int64_t)(k + u * KG) * g.ld);
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) v[u] = widen(x[(int64_t)(k + u * KG) * g.incx]);
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf(v[u], widen(m[u][e]), acc[e]);
            }
            for (; k < k1; k += KG) {
                const u16x8 m = load8(col + (int64_t)k * g.ld);
                const float v = widen(x[(int64_t)k * g.incx]);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf(v, widen(m[e]), acc[e]);
            }
            done = true;
        }
    }
    if (!done) {
        // element-wise: every lane of the unaligned variant, and the lane that straddles the last column otherwise
        for (int k = k0 + kg; k < k1; k += KG) {
            const float v = widen(x[(int64_t)k * g.incx]);
#pragma unroll
            for (int e = 0; e < PER; ++e)
                if (j + e < g.len) acc[e] = __builtin_fmaf(v, widen(col[(int64_t)k * g.ld + e]), acc[e]);
        }
    }
#pragma unroll
    for (int e = 0; e < PER; ++e) red[kg][cl * PER + e] = acc[e];
    __syncthreads();
    if (tid < CW && j0 + tid < g.len) {
        float s = red[0][tid];
        for (int q = 1; q < KG; ++q) s += red[q][tid];
        g.y[(int64_t)slice * g.slice_stride + (int64_t)(j0 + tid) * g.incy] = s;
    }
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

// as a profiler trace prints the kernels
const char *gemv_bf16_kernel_name(int pattern, bool vec)
{
    if (pattern == kVecRows) return vec ? "gemv_rows_bf16_kernel<true>" : "gemv_rows_bf16_kernel<false>";
    return vec ? "gemv_cols_bf16_kernel<true>" : "gemv_cols_bf16_kernel<false>";
}

bool gemv_bf16_takes_vectors(const VecArgs16 &a) { return aligned16(a.mat) && a.ld % 8 == 0; }

// len >= 1, K >= 1, k_slices >= 1; the number of workgroups must fit a grid (checked by the caller)
hipError_t launch_gemv_bf16(int pattern, VecArgs16 a, hipStream_t s)
{
    const bool vec = gemv_bf16_takes_vectors(a);
    a.xvec = a.incx == 1 && aligned16(a.x);
    if (pattern == kVecRows) {
        const dim3 grid((unsigned)((a.len + 3) / 4 * a.k_slices));
        if (vec) hipLaunchKernelGGL(gemv_rows_bf16_kernel<true>, grid, dim3(kThreads), 0, s, a);
        else hipLaunchKernelGGL(gemv_rows_bf16_kernel<false>, grid, dim3(kThreads), 0, s, a);
    } else {
        const dim3 grid((unsigned)((a.len + 63) / 64 * a.k_slices));
        if (vec) hipLaunchKernelGGL(gemv_cols_bf16_kernel<true>, grid, dim3(kThreads), 0, s, a);
        else hipLaunchKernelGGL(gemv_cols_bf16_kernel<false>, grid, dim3(kThreads), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace fsrgemm
