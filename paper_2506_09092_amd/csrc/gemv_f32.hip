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
// A few vectors on one side (2 .. 16 rows of A or columns of B, kMaxFewVectorsF32) stream the matrix once as well, every
// element now feeding one multiply-add per vector.  The two patterns keep their shape; what changes is that a
// workgroup stages its K range of the vectors through LDS (any strides on the global side, zeros behind the
// last vector and behind the K range), chunk by chunk in two buffers, one barrier per chunk, and requests a matrix
// piece of the next chunk as soon as the register of the current chunk's piece is free (a ring of loads):
//   rows:  a wavefront takes four matrix rows, two 16-byte pieces of each in flight per lane (512 k per chunk),
//          and reads the matching pieces of every vector from LDS; 4 x R sums per lane, butterflies at the end.
//   cols:  as above (32 columns, 32 groups of lanes, eight rows in flight), the vectors' elements of a matrix
//          row sit side by side in LDS and are read as 16-byte pieces; 4 x R sums per lane, added over a
//          wavefront's eight groups by lane exchange and over the four wavefronts through LDS, in fixed order.
// Any alignment of the matrix; the cols pattern needs at least four columns (gemv_takes_few).
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

// a 16-byte load from an address that is only element-aligned (allowed on this target)
typedef f32x4 f32x4_elem_aligned __attribute__((aligned(4)));
__device__ __forceinline__ f32x4 load4_any(const float *p) { return *reinterpret_cast<const f32x4_elem_aligned *>(p); }

// The K range [kc, kc + KC) of the R vectors on its way into LDS, in two steps so that the loads' latency passes
// behind other work: fetch_vectors reads a lane's share into registers, store_vectors writes it: element (k, r) to
// xs[k * R + r] (K_MAJOR) or xs[r * KC + k].  Lanes walk k fastest when the vectors are contiguous along k, r
// fastest otherwise, so that either storage is read in contiguous runs.  Zeros behind vector g.nvec - 1 and from k1
// on: every load is issued, from the last valid element where its own lies outside, and store_vectors replaces such
// values (no branch, and nothing that waits for a load, in the loops that call fetch_vectors).  k1 >= 1.
template <int R, int KC>
__device__ __forceinline__ void fetch_vectors(float (&xr)[R * KC / kThreads], const VecArgs &g, int kc, int k1)
{
    const int tid = threadIdx.x;
    const float *__restrict__ x = g.x;
    if (g.incx == 1) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int q = 0; q < KC / kThreads; ++q)
                xr[r * (KC / kThreads) + q] = x[(int64_t)min(kc + tid + q * kThreads, k1 - 1) + (int64_t)min(r, g.nvec - 1) * g.ldx];
    } else {
        const float *__restrict__ xl = x + (int64_t)min(tid % R, g.nvec - 1) * g.ldx;       // (kThreads is a multiple of R)
#pragma unroll
        for (int q = 0; q < R * KC / kThreads; ++q) xr[q] = xl[(int64_t)min(kc + tid / R + q * (kThreads / R), k1 - 1) * g.incx];
    }
}
template <int R, int KC, bool K_MAJOR>
__device__ __forceinline__ void store_vectors(float *__restrict__ xs, const float (&xr)[R * KC / kThreads], const VecArgs &g, int kc, int k1)
{
    const int tid = threadIdx.x;
    if (g.incx == 1) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int q = 0; q < KC / kThreads; ++q) {
                const int kl = tid + q * kThreads;
                xs[K_MAJOR ? kl * R + r : r * KC + kl] = r < g.nvec && kc + kl < k1 ? xr[r * (KC / kThreads) + q] : 0.f;
            }
    } else {
        const int r = tid % R;
#pragma unroll
        for (int q = 0; q < R * KC / kThreads; ++q) {
            const int kl = tid / R + q * (kThreads / R);
            xs[K_MAJOR ? kl * R + r : r * KC + kl] = r < g.nvec && kc + kl < k1 ? xr[q] : 0.f;
        }
    }
}

// rows pattern, R vectors (g.nvec <= R): y_r[i] = sum_k Mat[i][k] x_r[k]; any alignment
template <int R>
__global__ __launch_bounds__(kThreads) void gemv_rows_f32_few_kernel(VecArgs g)
{
    constexpr int RW = 4, KC = 512;                           // matrix rows per wavefront, k per chunk
    __shared__ __attribute__((aligned(16))) float xs[2][R * KC];
    const int groups = (g.len + 4 * RW - 1) / (4 * RW);
    const int slice = (int)blockIdx.x / groups;
    const int row0 = ((int)blockIdx.x - slice * groups) * (4 * RW) + ((int)threadIdx.x >> 6) * RW;
    const int lane = threadIdx.x & 63;
    const int per = (((g.K + g.k_slices - 1) / g.k_slices) + 3) & ~3;     // slices start at multiples of 4: pieces of an aligned matrix stay aligned
    const int k0 = (int)min((int64_t)slice * per, (int64_t)g.K), k1 = (int)min((int64_t)k0 + per, (int64_t)g.K);
    const int k4 = k0 + ((k1 - k0) & ~3);                     // whole pieces up to here, up to three elements behind
    const float *__restrict__ rowp[RW];
#pragma unroll
    for (int i = 0; i < RW; ++i) rowp[i] = g.mat + (int64_t)min(row0 + i, g.len - 1) * g.ld;      // rows behind the last repeat it
    float acc[RW][R];
#pragma unroll
    for (int i = 0; i < RW; ++i)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[i][r] = 0.f;
    f32x4 m[RW][2];
    float xr[R * KC / kThreads];
    if (k0 < k4) {
        // pieces u of chunk kc, two per row and lane; in place of a piece that lies behind the whole pieces the slice's
        // first piece is read, and zeros are used
        auto fetch_rows = [&](int kc, int u) {
            const int k = kc + 4 * lane + 256 * u;
            const int kk = k < k4 ? k : k0;
#pragma unroll
            for (int i = 0; i < RW; ++i) m[i][u] = load4_any(rowp[i] + kk);
        };
        fetch_rows(k0, 0);
        fetch_rows(k0, 1);
        fetch_vectors<R, KC>(xr, g, k0, k4);
        store_vectors<R, KC, false>(xs[0], xr, g, k0, k4);
        __syncthreads();
        int buf = 0;
        // The registers of the matrix pieces are a ring: as soon as a piece has been used, the piece that takes its place
        // in the next chunk is requested, so all but the pieces in use are in flight all the time (behind the last
        // chunk the requests repeat the slice's first pieces and nothing uses them).  The next chunk's vector elements
        // are requested before the arithmetic and written to the other buffer behind it; one barrier per chunk.
        for (int kc = k0; kc < k4; kc += KC, buf ^= 1) {
            fetch_vectors<R, KC>(xr, g, kc + KC, k4);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const bool in = kc + 4 * lane + 256 * u < k4;
                f32x4 mm[RW];
#pragma unroll
                for (int i = 0; i < RW; ++i)
#pragma unroll
                    for (int e = 0; e < 4; ++e) mm[i][e] = in ? m[i][u][e] : 0.f;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const f32x4 v = *reinterpret_cast<const f32x4 *>(&xs[buf][r * KC + 4 * lane + 256 * u]);
#pragma unroll
                    for (int i = 0; i < RW; ++i) acc[i][r] = dot4(mm[i], v, acc[i][r]);
                }
                fetch_rows(kc + KC, u);
            }
            store_vectors<R, KC, false>(xs[buf ^ 1], xr, g, kc + KC, k4);
            __syncthreads();
        }
    }
    if (lane < k1 - k4) {                                     // the up to three elements behind the last whole piece
        const int k = k4 + lane;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float v = r < g.nvec ? g.x[(int64_t)k * g.incx + (int64_t)r * g.ldx] : 0.f;
#pragma unroll
            for (int i = 0; i < RW; ++i) acc[i][r] = __builtin_fmaf(rowp[i][k], v, acc[i][r]);
        }
    }
#pragma unroll
    for (int i = 0; i < RW; ++i)
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float s = acc[i][r];
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d, 64);
            if (lane == 0 && row0 + i < g.len && r < g.nvec)
                g.y[(int64_t)slice * g.slice_stride + (int64_t)(row0 + i) * g.incy + (int64_t)r * g.ldy] = s;
        }
}

// cols pattern, R vectors (g.nvec <= R): y_r[j] = sum_k x_r[k] Mat[k][j]; requires gemv_takes_few(kVecCols, g): any alignment
template <int R>
__global__ __launch_bounds__(kThreads) void gemv_cols_f32_few_kernel(VecArgs g)
{
    constexpr int CW = 32, LANES = 8, KG = kThreads / LANES, UNROLL = 8, KC = KG * UNROLL;
    __shared__ __attribute__((aligned(16))) float xs[2][KC * R];
    __shared__ float red[kThreads / 64][R][CW];
    const int groups = (g.len + CW - 1) / CW;
    const int slice = (int)blockIdx.x / groups;
    const int j0 = ((int)blockIdx.x - slice * groups) * CW;
    const int tid = threadIdx.x, cl = tid % LANES, kg = tid / LANES;
    const int per = (g.K + g.k_slices - 1) / g.k_slices;
    const int k0 = (int)min((int64_t)slice * per, (int64_t)g.K), k1 = (int)min((int64_t)k0 + per, (int64_t)g.K);
    // a lane whose four columns straddle or lie behind the last one takes the matrix's last four instead: it repeats
    // sums that other lanes of its group form from the same values in the same order
    const int j = min(j0 + cl * 4, g.len - 4);
    const float *__restrict__ col = g.mat + j;
    float acc[R][4];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[r][e] = 0.f;
    f32x4 m[UNROLL];
    float xr[R * KC / kThreads];
    if (k0 < k1) {
        // piece u of chunk kc: matrix row kc + kg + 32 u; behind the K range the range's last row is read, and zeros are used
        auto fetch_cols = [&](int kc, int u) { m[u] = load4_any(col + (int64_t)min(kc + kg + u * KG, k1 - 1) * g.ld); };
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) fetch_cols(k0, u);
        fetch_vectors<R, KC>(xr, g, k0, k1);
        store_vectors<R, KC, true>(xs[0], xr, g, k0, k1);
        __syncthreads();
        int buf = 0;
        // The registers of the matrix pieces are a ring: as soon as a piece has been used, the piece that takes its place
        // in the next chunk is requested, so all but the piece in use are in flight all the time (behind the last chunk
        // the requests repeat the range's last row and nothing uses them).  The next chunk's vector elements are
        // requested before the arithmetic and written to the other buffer behind it; one barrier per chunk.
        for (int kc = k0; kc < k1; kc += KC, buf ^= 1) {
            fetch_vectors<R, KC>(xr, g, kc + KC, k1);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const float *xk = &xs[buf][(kg + u * KG) * R];
                float v[R];
                if constexpr (R % 4 == 0) {
#pragma unroll
                    for (int q = 0; q < R / 4; ++q) {
                        const f32x4 t = *reinterpret_cast<const f32x4 *>(xk + 4 * q);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[4 * q + e] = t[e];
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < R; ++r) v[r] = xk[r];
                }
                const bool in = kc + kg + u * KG < k1;
                f32x4 mm;
#pragma unroll
                for (int e = 0; e < 4; ++e) mm[e] = in ? m[u][e] : 0.f;
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[r][e] = __builtin_fmaf(v[r], mm[e], acc[r][e]);
                fetch_cols(kc + KC, u);
            }
            store_vectors<R, KC, true>(xs[buf ^ 1], xr, g, kc + KC, k1);
            __syncthreads();
        }
    }
    // the eight groups of a wavefront by lane exchange (8, 16, 32 lanes apart), then the four wavefronts in order
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float s = acc[r][e];
            s += __shfl_xor(s, 8, 64);
            s += __shfl_xor(s, 16, 64);
            s += __shfl_xor(s, 32, 64);
            const int c = j + e - j0;                         // (negative where the last four columns begin in the group before)
            if ((tid & 63) < LANES && c >= 0) red[tid >> 6][r][c] = s;
        }
    __syncthreads();
    for (int o = tid; o < R * CW; o += kThreads) {
        const int r = o / CW, c = o % CW;
        if (r < g.nvec && j0 + c < g.len) {
            float s = red[0][r][c];
            for (int q = 1; q < kThreads / 64; ++q) s += red[q][r][c];
            g.y[(int64_t)slice * g.slice_stride + (int64_t)(j0 + c) * g.incy + (int64_t)r * g.ldy] = s;
        }
    }
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <int R>
void launch_few(int pattern, const VecArgs &a, hipStream_t s)
{
    if (pattern == kVecRows) hipLaunchKernelGGL(gemv_rows_f32_few_kernel<R>, dim3((unsigned)((a.len + 15) / 16 * a.k_slices)), dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL(gemv_cols_f32_few_kernel<R>, dim3((unsigned)((a.len + 31) / 32 * a.k_slices)), dim3(kThreads), 0, s, a);
}

}  // namespace

// as a profiler trace prints the kernels
const char *gemv_kernel_name(int pattern, bool vec, int nvec)
{
    if (nvec > 1) {
        if (pattern == kVecRows) return nvec <= 2 ? "gemv_rows_f32_few_kernel<2>" : nvec <= 4 ? "gemv_rows_f32_few_kernel<4>" : nvec <= 8 ? "gemv_rows_f32_few_kernel<8>" : "gemv_rows_f32_few_kernel<16>";
        return nvec <= 2 ? "gemv_cols_f32_few_kernel<2>" : nvec <= 4 ? "gemv_cols_f32_few_kernel<4>" : nvec <= 8 ? "gemv_cols_f32_few_kernel<8>" : "gemv_cols_f32_few_kernel<16>";
    }
    if (pattern == kVecRows) return vec ? "gemv_rows_f32_kernel<true>" : "gemv_rows_f32_kernel<false>";
    return vec ? "gemv_cols_f32_kernel<true>" : "gemv_cols_f32_kernel<false>";
}

bool gemv_takes_vectors(const VecArgs &a) { return aligned16(a.mat) && a.ld % 4 == 0; }
// the kernels for several vectors: any alignment (their 16-byte loads are issued from element-aligned addresses); the
// cols pattern needs at least one whole piece of columns
bool gemv_takes_few(int pattern, const VecArgs &a) { return pattern == kVecRows || a.len >= 4; }

// len >= 1, K >= 1, k_slices >= 1; the number of workgroups must fit a grid (checked by the caller); more than one
// vector only on a matrix of aligned pieces
hipError_t launch_gemv_f32(int pattern, VecArgs a, hipStream_t s)
{
    const bool vec = gemv_takes_vectors(a);
    if (a.nvec < 1 || a.nvec > kMaxFewVectorsF32 || (a.nvec > 1 && !gemv_takes_few(pattern, a))) return hipErrorInvalidValue;
    if (a.nvec > 1) {
        if (a.nvec <= 2) launch_few<2>(pattern, a, s);
        else if (a.nvec <= 4) launch_few<4>(pattern, a, s);
        else if (a.nvec <= 8) launch_few<8>(pattern, a, s);
        else launch_few<16>(pattern, a, s);
        return hipGetLastError();
    }
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
