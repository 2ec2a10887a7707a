// fp32 products in which M or N is 1 (the paper's Task 2 with a vector on one side): y = Mat . x or
// y = x . Mat.  Every matrix element is used once, so the matrix streams from HBM exactly once and bandwidth
// bounds the kernel; the matrix cores have nothing to reuse and are not involved.  Two access patterns cover
// the four storage cases:
//   rows:  the matrix is contiguous along the summation index, y[r] = sum_k Mat[r][k] x[k]
//          (row-major A times a column, or a row times a B stored transposed).  One wavefront per row: its
//          lanes read 16-byte pieces 1 KB apart in steps of 256 elements, four in flight, multiply by the matching
//          piece of x (served from cache) and the 64 partial sums are added in a fixed butterfly.
//   cols:  the matrix is contiguous along the output index, y[j] = sum_k x[k] Mat[k][j]
//          (a row times a row-major B, or an A stored transposed times a column).  One workgroup per 32
//          output columns (one 128-byte line of every matrix row): 8 lanes cover the line, 32 groups of lanes
//          take every 32nd row, eight rows in flight each, and the 32 partial sums per column are added in
//          group order through LDS.
// With k_slices > 1 the K range is cut into slices, workgroup ids beyond the first round belong to further
// slices and every slice writes its partial y to its own vector behind g.y (a workspace); the caller adds the
// slices with the split-K reduction kernel.  All sums have a fixed order: results repeat bit for bit.
#include "launchers.hpp"

namespace fsrgemm {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ f32x4 load4(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }

// x[k .. k + 3], as one vector when x is contiguous and 16-byte aligned
__device__ __forceinline__ f32x4 load_x4(const float *x, int64_t incx, bool xvec, int k)
{
    if (xvec) return load4(x + k);
    f32x4 v;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = x[(int64_t)(k + e) * incx];
    return v;
}

__device__ __forceinline__ float dot4(f32x4 a, f32x4 b, float acc)
{
#pragma unroll
    for (int e = 0; e < 4; ++e) acc = __builtin_fmaf(a[e], b[e], acc);
    return acc;
}

// VEC: the matrix base is 16-byte aligned and ld a multiple of 4, so 16-byte loads of whole pieces are aligned
template <bool VEC>
__global__ __launch_bounds__(kThreads) void gemv_rows_f32_kernel(VecArgs g)
{
    const int groups = (g.len + 3) / 4;                       // four rows per workgroup, one per wavefront
    const int slice = (int)blockIdx.x / groups;
    const int r = ((int)blockIdx.x - slice * groups) * 4 + ((int)threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (r >= g.len) return;
    // slices start at multiples of 4 so that vector loads stay aligned
    const int per = (((g.K + g.k_slices - 1) / g.k_slices) + 3) & ~3;
    const int k0 = min((int64_t)slice * per, (int64_t)g.K), k1 = min((int64_t)k0 + per, (int64_t)g.K);
    const float *__restrict__ row = g.mat + (int64_t)r * g.ld;
    const float *__restrict__ x = g.x;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    if constexpr (VEC) {
        int k = k0 + 4 * lane;
        for (; k + 771 < k1; k += 1024) {
            f32x4 m[4], v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) m[u] = load4(row + k + 256 * u);
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = load_x4(x, g.incx, g.xvec, k + 256 * u);
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] = dot4(m[u], v[u], acc[u]);
        }
        for (; k + 3 < k1; k += 256) acc[0] = dot4(load4(row + k), load_x4(x, g.incx, g.xvec, k), acc[0]);
        const int kt = k0 + ((k1 - k0) & ~3) + lane;           // the up to three elements behind the last whole piece
        if (lane < ((k1 - k0) & 3)) acc[1] = __builtin_fmaf(row[kt], x[(int64_t)kt * g.incx], acc[1]);
    } else {
        int k = k0 + lane;
        for (; k + 192 < k1; k += 256) {
            float m[4], v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) m[u] = row[k + 64 * u];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = x[(int64_t)(k + 64 * u) * g.incx];
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[u] = __builtin_fmaf(m[u], v[u], acc[u]);
        }
        for (; k < k1; k += 64) acc[0] = __builtin_fmaf(row[k], x[(int64_t)k * g.incx], acc[0]);
    }
    float s = (acc[0] + acc[1]) + (acc[2] + acc[3]);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d, 64);
    if (lane == 0) g.y[(int64_t)slice * g.slice_stride + (int64_t)r * g.incy] = s;
}

template <bool VEC>
__global__ __launch_bounds__(kThreads) void gemv_cols_f32_kernel(VecArgs g)
{
    constexpr int CW = 32;                                    // output columns per workgroup
    constexpr int LANES = VEC ? 8 : 32, PER = CW / LANES;     // lanes across the columns, columns per lane
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
    const float *__restrict__ col = g.mat + j;
    const float *__restrict__ x = g.x;
    float acc[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) acc[e] = 0.f;

    bool done = false;
    if constexpr (VEC) {
        if (j + 3 < g.len) {
            int k = k0 + kg;
            for (; k + (UNROLL - 1) * KG < k1; k += UNROLL * KG) {
                f32x4 m[UNROLL];
                float v[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) m[u] = load4(col + (int64_t)(k + u * KG) * g.ld);
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) v[u] = x[(int64_t)(k + u * KG) * g.incx];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[e] = __builtin_fmaf(v[u], m[u][e], acc[e]);
            }
            for (; k < k1; k += KG) {
                const f32x4 m = load4(col + (int64_t)k * g.ld);
                const float v = x[(int64_t)k * g.incx];
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] = __builtin_fmaf(v, m[e], acc[e]);
            }
            done = true;
        }
    }
    if (!done) {
        // element-wise: every lane of the unaligned variant, and the lane that straddles the last column otherwise
        for (int k = k0 + kg; k < k1; k += KG) {
            const float v = x[(int64_t)k * g.incx];
#pragma unroll
            for (int e = 0; e < PER; ++e)
                if (j + e < g.len) acc[e] = __builtin_fmaf(v, col[(int64_t)k * g.ld + e], acc[e]);
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
const char *gemv_kernel_name(int pattern, bool vec)
{
    if (pattern == kVecRows) return vec ? "gemv_rows_f32_kernel<true>" : "gemv_rows_f32_kernel<false>";
    return vec ? "gemv_cols_f32_kernel<true>" : "gemv_cols_f32_kernel<false>";
}

bool gemv_takes_vectors(const VecArgs &a) { return aligned16(a.mat) && a.ld % 4 == 0; }

// len >= 1, K >= 1, k_slices >= 1; the number of workgroups must fit a grid (checked by the caller)
hipError_t launch_gemv_f32(int pattern, VecArgs a, hipStream_t s)
{
    const bool vec = gemv_takes_vectors(a);
    a.xvec = a.incx == 1 && aligned16(a.x);
    if (pattern == kVecRows) {
        const dim3 grid((unsigned)((a.len + 3) / 4 * a.k_slices));
        if (vec) hipLaunchKernelGGL(gemv_rows_f32_kernel<true>, grid, dim3(kThreads), 0, s, a);
        else hipLaunchKernelGGL(gemv_rows_f32_kernel<false>, grid, dim3(kThreads), 0, s, a);
    } else {
        const dim3 grid((unsigned)((a.len + 31) / 32 * a.k_slices));
        if (vec) hipLaunchKernelGGL(gemv_cols_f32_kernel<true>, grid, dim3(kThreads), 0, s, a);
        else hipLaunchKernelGGL(gemv_cols_f32_kernel<false>, grid, dim3(kThreads), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace fsrgemm
