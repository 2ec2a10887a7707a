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
// A few vectors on one side (2 .. 8 rows of A or columns of B, kMaxFewVectors) go the way they go in fp32: the
// workgroup stages its K range of the vectors through LDS (as bf16, any strides on the global side, zeros behind
// the last vector and behind the K range), chunk by chunk in two buffers with one barrier per chunk; the registers of
// the matrix pieces are a ring (a register's next content is requested as soon as its current content has been
// used); no branch in the loops, and no value replaced right behind its load: pieces outside the K range or the
// matrix are read from a valid place and replaced by zeros where they are used.
//   rows:  a wavefront takes four matrix rows, two pieces of each in flight per lane (1024 k per chunk).
//   cols:  64 columns, 32 groups of lanes, eight rows in flight each (256 k per chunk); the vectors' elements of
//          a matrix row sit side by side in LDS; the sums of a wavefront's eight groups are added by lane exchange,
//          the four wavefronts' through LDS, in fixed order.
// Any alignment of the matrix; the cols pattern needs at least eight columns (gemv_bf16_takes_few).
// Where vectors and matrix are both contiguous along k, aligned, and K is whole 16-byte pieces, up to 16 vectors go
// through the matrix cores instead (gemv_rows_bf16_mfma_direct_kernel, gemv_rows_bf16_mfma_kernel, described where
// they stand).
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

// a 16-byte load from an address that is only element-aligned (allowed on this target)
typedef u16x8 u16x8_elem_aligned __attribute__((aligned(2)));
__device__ __forceinline__ u16x8 load8_any(const uint16_t *p) { return *reinterpret_cast<const u16x8_elem_aligned *>(p); }

// The K range [kc, kc + KC) of the R vectors on its way into LDS, in two steps so that the loads' latency passes
// behind other work: fetch_vectors reads a lane's share into registers, store_vectors writes it: element (k, r) to
// xs[k * R + r] (K_MAJOR) or xs[r * KC + k].  Lanes walk k fastest when the vectors are contiguous along k, r
// fastest otherwise.  Every load is issued, from the last valid element where its own lies outside (behind vector
// g.nvec - 1, from k1 on), and store_vectors writes zeros for those.  k1 >= 1.
template <int R, int KC>
__device__ __forceinline__ void fetch_vectors(uint16_t (&xr)[R * KC / kThreads], const VecArgs16 &g, int kc, int k1)
{
    const int tid = threadIdx.x;
    const uint16_t *__restrict__ x = g.x;
    if (g.incx == 1) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int q = 0; q < KC / kThreads; ++q)
                xr[r * (KC / kThreads) + q] = x[(int64_t)min(kc + tid + q * kThreads, k1 - 1) + (int64_t)min(r, g.nvec - 1) * g.ldx];
    } else {
        const uint16_t *__restrict__ xl = x + (int64_t)min(tid % R, g.nvec - 1) * g.ldx;    // (kThreads is a multiple of R)
#pragma unroll
        for (int q = 0; q < R * KC / kThreads; ++q) xr[q] = xl[(int64_t)min(kc + tid / R + q * (kThreads / R), k1 - 1) * g.incx];
    }
}
template <int R, int KC, bool K_MAJOR>
__device__ __forceinline__ void store_vectors(uint16_t *__restrict__ xs, const uint16_t (&xr)[R * KC / kThreads], const VecArgs16 &g, int kc, int k1)
{
    const int tid = threadIdx.x;
    if (g.incx == 1) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int q = 0; q < KC / kThreads; ++q) {
                const int kl = tid + q * kThreads;
                xs[K_MAJOR ? kl * R + r : r * KC + kl] = r < g.nvec && kc + kl < k1 ? xr[r * (KC / kThreads) + q] : (uint16_t)0;
            }
    } else {
        const int r = tid % R;
#pragma unroll
        for (int q = 0; q < R * KC / kThreads; ++q) {
            const int kl = tid / R + q * (kThreads / R);
            xs[K_MAJOR ? kl * R + r : r * KC + kl] = r < g.nvec && kc + kl < k1 ? xr[q] : (uint16_t)0;
        }
    }
}

// rows pattern, R vectors (g.nvec <= R): y_r[i] = sum_k Mat[i][k] x_r[k]; any alignment
template <int R>
__global__ __launch_bounds__(kThreads) void gemv_rows_bf16_few_kernel(VecArgs16 g)
{
    constexpr int RW = 4, KC = 1024;                          // matrix rows per wavefront, k per chunk
    __shared__ __attribute__((aligned(16))) uint16_t xs[2][R * KC];
    const int groups = (g.len + 4 * RW - 1) / (4 * RW);
    const int slice = (int)blockIdx.x / groups;
    const int row0 = ((int)blockIdx.x - slice * groups) * (4 * RW) + ((int)threadIdx.x >> 6) * RW;
    const int lane = threadIdx.x & 63;
    const int per = (((g.K + g.k_slices - 1) / g.k_slices) + 7) & ~7;     // slices start at multiples of 8: pieces stay aligned
    const int k0 = (int)min((int64_t)slice * per, (int64_t)g.K), k1 = (int)min((int64_t)k0 + per, (int64_t)g.K);
    const int k8 = k0 + ((k1 - k0) & ~7);                     // whole pieces up to here, up to seven elements behind
    const uint16_t *__restrict__ rowp[RW];
#pragma unroll
    for (int i = 0; i < RW; ++i) rowp[i] = g.mat + (int64_t)min(row0 + i, g.len - 1) * g.ld;      // rows behind the last repeat it
    float acc[RW][R];
#pragma unroll
    for (int i = 0; i < RW; ++i)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[i][r] = 0.f;
    u16x8 m[RW][2];
    uint16_t xr[R * KC / kThreads];
    if (k0 < k8) {
        // pieces u of chunk kc, two per row and lane; in place of a piece that lies behind the whole pieces the slice's
        // first piece is read, and zeros are used
        auto fetch_rows = [&](int kc, int u) {
            const int k = kc + 8 * lane + 512 * u;
            const int kk = k < k8 ? k : k0;
#pragma unroll
            for (int i = 0; i < RW; ++i) m[i][u] = load8_any(rowp[i] + kk);
        };
        fetch_rows(k0, 0);
        fetch_rows(k0, 1);
        fetch_vectors<R, KC>(xr, g, k0, k8);
        store_vectors<R, KC, false>(xs[0], xr, g, k0, k8);
        __syncthreads();
        int buf = 0;
        for (int kc = k0; kc < k8; kc += KC, buf ^= 1) {
            fetch_vectors<R, KC>(xr, g, kc + KC, k8);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const bool in = kc + 8 * lane + 512 * u < k8;
                float mm[RW][8];
#pragma unroll
                for (int i = 0; i < RW; ++i)
#pragma unroll
                    for (int e = 0; e < 8; ++e) mm[i][e] = in ? widen(m[i][u][e]) : 0.f;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const u16x8 v = *reinterpret_cast<const u16x8 *>(&xs[buf][r * KC + 8 * lane + 512 * u]);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float ve = widen(v[e]);
#pragma unroll
                        for (int i = 0; i < RW; ++i) acc[i][r] = __builtin_fmaf(mm[i][e], ve, acc[i][r]);
                    }
                }
                fetch_rows(kc + KC, u);
            }
            store_vectors<R, KC, false>(xs[buf ^ 1], xr, g, kc + KC, k8);
            __syncthreads();
        }
    }
    if (lane < k1 - k8) {                                     // the up to seven elements behind the last whole piece
        const int k = k8 + lane;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float v = r < g.nvec ? widen(g.x[(int64_t)k * g.incx + (int64_t)r * g.ldx]) : 0.f;
#pragma unroll
            for (int i = 0; i < RW; ++i) acc[i][r] = __builtin_fmaf(widen(rowp[i][k]), v, acc[i][r]);
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

// cols pattern, R vectors (g.nvec <= R): y_r[j] = sum_k x_r[k] Mat[k][j]; requires gemv_bf16_takes_few(kVecCols, g)
template <int R>
__global__ __launch_bounds__(kThreads) void gemv_cols_bf16_few_kernel(VecArgs16 g)
{
    constexpr int CW = 64, LANES = 8, KG = kThreads / LANES, UNROLL = 8, KC = KG * UNROLL;
    __shared__ __attribute__((aligned(16))) uint16_t xs[2][KC * R];
    __shared__ float red[kThreads / 64][R][CW];
    const int groups = (g.len + CW - 1) / CW;
    const int slice = (int)blockIdx.x / groups;
    const int j0 = ((int)blockIdx.x - slice * groups) * CW;
    const int tid = threadIdx.x, cl = tid % LANES, kg = tid / LANES;
    const int per = (g.K + g.k_slices - 1) / g.k_slices;
    const int k0 = (int)min((int64_t)slice * per, (int64_t)g.K), k1 = (int)min((int64_t)k0 + per, (int64_t)g.K);
    // a lane whose eight columns straddle or lie behind the last one takes the matrix's last eight instead: it repeats
    // sums that other lanes of its group form from the same values in the same order
    const int j = min(j0 + cl * 8, g.len - 8);
    const uint16_t *__restrict__ col = g.mat + j;
    float acc[R][8];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] = 0.f;
    u16x8 m[UNROLL];
    uint16_t xr[R * KC / kThreads];
    if (k0 < k1) {
        // piece u of chunk kc: matrix row kc + kg + 32 u; behind the K range the range's last row is read, and zeros are used
        auto fetch_cols = [&](int kc, int u) { m[u] = load8_any(col + (int64_t)min(kc + kg + u * KG, k1 - 1) * g.ld); };
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) fetch_cols(k0, u);
        fetch_vectors<R, KC>(xr, g, k0, k1);
        store_vectors<R, KC, true>(xs[0], xr, g, k0, k1);
        __syncthreads();
        int buf = 0;
        for (int kc = k0; kc < k1; kc += KC, buf ^= 1) {
            fetch_vectors<R, KC>(xr, g, kc + KC, k1);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint16_t *xk = &xs[buf][(kg + u * KG) * R];
                typedef uint16_t u16xR __attribute__((ext_vector_type(R)));
                const u16xR xv = *reinterpret_cast<const u16xR *>(xk);       // (R elements of 2 bytes at a multiple of 2 R bytes)
                float v[R];
#pragma unroll
                for (int r = 0; r < R; ++r) v[r] = widen(xv[r]);
                const bool in = kc + kg + u * KG < k1;
                float mm[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) mm[e] = in ? widen(m[u][e]) : 0.f;
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[r][e] = __builtin_fmaf(v[r], mm[e], acc[r][e]);
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
        for (int e = 0; e < 8; ++e) {
            float s = acc[r][e];
            s += __shfl_xor(s, 8, 64);
            s += __shfl_xor(s, 16, 64);
            s += __shfl_xor(s, 32, 64);
            const int c = j + e - j0;                         // (negative where the last eight columns begin in the group before)
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

// rows pattern on the matrix cores, up to 16 vectors that are contiguous along k (kMaxMfmaVectors; the storage gemm_bf16
// takes: a few rows of a row-major A against a column-major B, or a row-major A against a few columns of such a B):
// y_r[i] = sum_k Mat[i][k] x_r[k] as D = X . Mat^T in steps of v_mfma_f32_16x16x32_bf16, so that the arithmetic no
// longer occupies the vector units.  Both fragments of that instruction are 16-byte pieces of memory as it lies: lane l
// holds the 8 values k = 8 (l / 16) .. + 7 of row l % 16 of its operand, and register r of the result holds row
// 4 (l / 16) + r of the first operand against row l % 16 of the second.
// Read that way, one load instruction fetches 64 bytes of each of 16 matrix rows (the kernel below does).  Here the 16
// columns of the second operand are 8 matrix rows times the two halves of a 128-byte line instead -- lane l reads piece
// 4 (l % 2) + l / 16 of the line of row (l % 16) / 2: one instruction, 8 whole lines, and a wavefront's 8 rows leave a
// workgroup of four wavefronts 32 rows over one K range -- and a step of 64 k takes two MFMAs on the same matrix fragment: one with the vectors' pieces 0 .. 3
// (its columns with l % 2 == 0 are products of matching k, the others are not and are never read), one with pieces
// 4 .. 7 (the other way round).  At the end the two halves of a row are added.
// A workgroup takes 32 matrix rows, 8 per wavefront, all over the same K range; the vectors' elements of a chunk of
// 1024 k go through LDS (read from global memory as whole rows of 1 KB, once per workgroup; two buffers, one barrier per
// chunk; rows padded by 16 bytes so that the 16 lanes of a fragment read hit different banks), and the 16 matrix
// pieces of a chunk are a ring of loads as above (a ring over two chunks, 32 KB per wavefront in flight, was no faster).  Pieces outside the K range are read from its first piece and
// replaced by zeros where they are used, vectors behind the last are zeros in LDS, matrix rows behind the last repeat
// the last.  Requires gemv_bf16_takes_mfma(g).
__global__ __launch_bounds__(kThreads) void gemv_rows_bf16_mfma_kernel(VecArgs16 g)
{
    constexpr int STEPS = 16, KC = 64 * STEPS, XROW = KC + 8;              // steps of 64 k per chunk; LDS row of a vector, in elements
    constexpr int XPER = 16 * (KC / 8) / kThreads;                         // 16-byte pieces of the vectors per lane and chunk
    __shared__ __attribute__((aligned(16))) uint16_t xs[2][16 * XROW];
    __shared__ float red[kThreads / 64][16][17];
    const int groups = (g.len + 31) / 32;
    const int slice = (int)blockIdx.x / groups;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int row0 = ((int)blockIdx.x - slice * groups) * 32 + 8 * wave;
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
    const int per = (((g.K + g.k_slices - 1) / g.k_slices) + 7) & ~7;     // slices start at multiples of 8: pieces stay aligned
    const int k0 = (int)min((int64_t)slice * per, (int64_t)g.K), k1 = (int)min((int64_t)k0 + per, (int64_t)g.K);
    const int piece = 4 * (l16 & 1) + lq;                                  // the lane's piece of a 128-byte line
    const uint16_t *__restrict__ mp = g.mat + (int64_t)min(row0 + (l16 >> 1), g.len - 1) * g.ld;
    f32x4 acc_lo = {0.f, 0.f, 0.f, 0.f}, acc_hi = {0.f, 0.f, 0.f, 0.f};     // against the vectors' pieces 0 .. 3 / 4 .. 7
    u16x8 m[STEPS], xr[XPER];
    if (k0 < k1) {
        // the lane's share of the vectors' chunk: piece tid % 128 of vector tid / 128 + 2 q
        auto fetch_x = [&](int kc) {
#pragma unroll
            for (int q = 0; q < XPER; ++q) {
                const int k = kc + 8 * (tid % (KC / 8));
                xr[q] = load8(g.x + (int64_t)min(tid / (KC / 8) + (kThreads / (KC / 8)) * q, g.nvec - 1) * g.ldx + (k < k1 ? k : k0));
            }
        };
        auto store_x = [&](uint16_t *dst, int kc) {
#pragma unroll
            for (int q = 0; q < XPER; ++q) {
                const int v = tid / (KC / 8) + (kThreads / (KC / 8)) * q, kl = 8 * (tid % (KC / 8));
                const bool in = v < g.nvec && kc + kl < k1;
                u16x8 t;
#pragma unroll
                for (int e = 0; e < 8; ++e) t[e] = in ? xr[q][e] : (uint16_t)0;
                *reinterpret_cast<u16x8 *>(dst + v * XROW + kl) = t;
            }
        };
        // step u of the chunk that begins at kc: the lane's piece of the line at k = kc + 64 u
        auto fetch_m = [&](int kc, int u) {
            const int k = kc + 64 * u + 8 * piece;
            m[u] = load8(mp + (k < k1 ? k : k0));
            // the load stays here, between the step before and the step behind: without the fence the compiler moves it
            // down to its use, and without the tie to the sums it moves all the steps ahead of all the loads
            asm volatile("" : "+v"(acc_lo) : : "memory");
        };
#pragma unroll
        for (int u = 0; u < STEPS; ++u) fetch_m(k0, u);
        fetch_x(k0);
        store_x(xs[0], k0);
        __syncthreads();
        int buf = 0;
        for (int kc = k0; kc < k1; kc += KC, buf ^= 1) {
            fetch_x(kc + KC);
#pragma unroll
            for (int u = 0; u < STEPS; ++u) {
                const uint16_t *xk = &xs[buf][l16 * XROW + 64 * u + 8 * lq];
                const u16x8 x_lo = *reinterpret_cast<const u16x8 *>(xk), x_hi = *reinterpret_cast<const u16x8 *>(xk + 32);
                const bool in = kc + 64 * u + 8 * piece < k1;
                u16x8 mm;
#pragma unroll
                for (int e = 0; e < 8; ++e) mm[e] = in ? m[u][e] : (uint16_t)0;
                acc_hi = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x_hi), __builtin_bit_cast(bf16x8, mm), acc_hi, 0, 0, 0);
                acc_lo = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x_lo), __builtin_bit_cast(bf16x8, mm), acc_lo, 0, 0, 0);
                fetch_m(kc + KC, u);
            }
            store_x(xs[buf ^ 1], kc + KC);
            __syncthreads();
        }
    }
    // column l % 16 of a lane is matrix row (l % 16) / 2 against the half l % 2 of its lines: that half's sums are valid
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave][l16][4 * lq + r] = (l16 & 1) ? acc_hi[r] : acc_lo[r];
    __syncthreads();
    for (int o = tid; o < 32 * 16; o += kThreads) {
        const int w = o / 128, rho = (o / 16) % 8, v = o % 16, row = row0 - 8 * wave + 8 * w + rho;
        if (v < g.nvec && row < g.len)
            g.y[(int64_t)slice * g.slice_stride + (int64_t)row * g.incy + (int64_t)v * g.ldy] = red[w][2 * rho][v] + red[w][2 * rho + 1][v];
    }
}

// The same product for up to kMfmaDirectVectors vectors, without LDS and without a barrier in the loop: both fragments
// come straight from global memory in the instruction's own layout (lane l: the 8 values k = 8 (l / 16) .. + 7 of row
// l % 16 of its operand, 16 matrix rows per workgroup, one MFMA per step of 32 k), the four wavefronts take a quarter
// of the K range each in blocks of 256 k = eight steps whose 16 loads are the ring, and the four partial blocks are added
// through LDS in wavefront order.  Every workgroup reads the vectors' whole K range from the L2 (with 16 vectors as many
// bytes as its share of the matrix), which is what this form costs as the vectors get more: 2 x 8192 x 8192 runs in
// 23 us, 8 x ... in 27.5, 16 x ... in 33, against 30 - 31 us for any number of vectors in the kernel above, which reads
// them once per 32 rows and in whole lines; on 16 x 28672 x 8192 it is 135 us against 110.  (A form with the matrix read
// in whole lines as above but the vectors still straight from memory, 8 rows per workgroup, was slower than both.)
__global__ __launch_bounds__(kThreads) void gemv_rows_bf16_mfma_direct_kernel(VecArgs16 g)
{
    constexpr int STEPS = 8, BLOCK = 32 * STEPS;
    __shared__ float red[kThreads / 64][16][17];
    const int groups = (g.len + 15) / 16;
    const int slice = (int)blockIdx.x / groups;
    const int row0 = ((int)blockIdx.x - slice * groups) * 16;
    const int lane = threadIdx.x & 63, l16 = lane & 15, lq = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);      // (a scalar: the K loop below is uniform)
    const int per = (((g.K + g.k_slices - 1) / g.k_slices) + 7) & ~7;     // slices start at multiples of 8: pieces stay aligned
    const int k0 = (int)min((int64_t)slice * per, (int64_t)g.K), k1 = (int)min((int64_t)k0 + per, (int64_t)g.K);
    const uint16_t *__restrict__ mp = g.mat + (int64_t)min(row0 + l16, g.len - 1) * g.ld;
    const uint16_t *__restrict__ xp = g.x + (int64_t)min(l16, g.nvec - 1) * g.ldx;
    const bool vec_in = l16 < g.nvec;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    u16x8 m[STEPS], x[STEPS];
    // the wavefront's quarter of the K range, in whole blocks
    const int quarter = ((k1 - k0 + 4 * BLOCK - 1) / (4 * BLOCK)) * BLOCK;
    const int w0 = k0 + wave * quarter, w1 = min(k1, w0 + quarter);
    if (w0 < w1) {
        // step u of the block that begins at kb: the lane's pieces at k = kb + 32 u + 8 (l / 16)
        auto fetch = [&](int kb, int u) {
            const int k = kb + 32 * u + 8 * lq;
            const int kk = k < w1 ? k : w0;
            m[u] = load8(mp + kk);
            x[u] = load8(xp + kk);
            // the loads stay here, between the step before and the step behind: without the fence the compiler moves them
            // down to their use, and without the tie to the sums it moves all the steps ahead of all the loads
            asm volatile("" : "+v"(acc) : : "memory");
        };
#pragma unroll
        for (int u = 0; u < STEPS; ++u) fetch(w0, u);
        for (int kb = w0; kb < w1; kb += BLOCK) {
#pragma unroll
            for (int u = 0; u < STEPS; ++u) {
                const bool in = kb + 32 * u + 8 * lq < w1;
                u16x8 mm, xx;
#pragma unroll
                for (int e = 0; e < 8; ++e) mm[e] = in ? m[u][e] : (uint16_t)0, xx[e] = in && vec_in ? x[u][e] : (uint16_t)0;
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xx), __builtin_bit_cast(bf16x8, mm), acc, 0, 0, 0);
                fetch(kb + BLOCK, u);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave][4 * lq + r][l16] = acc[r];
    __syncthreads();
    const int v = threadIdx.x >> 4, n = threadIdx.x & 15;
    if (v < g.nvec && row0 + n < g.len) {
        float s = red[0][v][n];
        for (int q = 1; q < kThreads / 64; ++q) s += red[q][v][n];
        g.y[(int64_t)slice * g.slice_stride + (int64_t)(row0 + n) * g.incy + (int64_t)v * g.ldy] = s;
    }
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <int R>
void launch_few(int pattern, const VecArgs16 &a, hipStream_t s)
{
    if (pattern == kVecRows) hipLaunchKernelGGL(gemv_rows_bf16_few_kernel<R>, dim3((unsigned)((a.len + 15) / 16 * a.k_slices)), dim3(kThreads), 0, s, a);
    else hipLaunchKernelGGL(gemv_cols_bf16_few_kernel<R>, dim3((unsigned)((a.len + 63) / 64 * a.k_slices)), dim3(kThreads), 0, s, a);
}

}  // namespace

// as a profiler trace prints the kernels
const char *gemv_bf16_kernel_name(int pattern, bool vec, int nvec, bool mfma)
{
    if (mfma) return nvec <= kMfmaDirectVectors ? "gemv_rows_bf16_mfma_direct_kernel" : "gemv_rows_bf16_mfma_kernel";
    if (nvec > 1) {
        if (pattern == kVecRows) return nvec <= 2 ? "gemv_rows_bf16_few_kernel<2>" : nvec <= 4 ? "gemv_rows_bf16_few_kernel<4>" : "gemv_rows_bf16_few_kernel<8>";
        return nvec <= 2 ? "gemv_cols_bf16_few_kernel<2>" : nvec <= 4 ? "gemv_cols_bf16_few_kernel<4>" : "gemv_cols_bf16_few_kernel<8>";
    }
    if (pattern == kVecRows) return vec ? "gemv_rows_bf16_kernel<true>" : "gemv_rows_bf16_kernel<false>";
    return vec ? "gemv_cols_bf16_kernel<true>" : "gemv_cols_bf16_kernel<false>";
}

bool gemv_bf16_takes_vectors(const VecArgs16 &a) { return aligned16(a.mat) && a.ld % 8 == 0; }
// the kernels for several vectors: any alignment (their 16-byte loads are issued from element-aligned addresses); the
// cols pattern needs at least one whole piece of columns
bool gemv_bf16_takes_few(int pattern, const VecArgs16 &a) { return pattern == kVecRows || a.len >= 8; }
// the matrix-core kernel: the rows pattern with 2 .. 16 vectors that are contiguous along k, everything in aligned
// pieces, K whole pieces
bool gemv_bf16_takes_mfma(int pattern, const VecArgs16 &a)
{
    return pattern == kVecRows && a.nvec >= 2 && a.nvec <= kMaxMfmaVectors && gemv_bf16_takes_vectors(a) && a.incx == 1 &&
           aligned16(a.x) && a.ldx % 8 == 0 && a.K % 8 == 0;
}

// len >= 1, K >= 1, k_slices >= 1; the number of workgroups must fit a grid (checked by the caller); more than one
// vector only on a matrix of aligned pieces
hipError_t launch_gemv_bf16(int pattern, VecArgs16 a, hipStream_t s)
{
    const bool vec = gemv_bf16_takes_vectors(a);
    if (gemv_bf16_takes_mfma(pattern, a)) {
        if (a.nvec <= kMfmaDirectVectors) hipLaunchKernelGGL(gemv_rows_bf16_mfma_direct_kernel, dim3((unsigned)((a.len + 15) / 16 * a.k_slices)), dim3(kThreads), 0, s, a);
        else hipLaunchKernelGGL(gemv_rows_bf16_mfma_kernel, dim3((unsigned)((a.len + 31) / 32 * a.k_slices)), dim3(kThreads), 0, s, a);
        return hipGetLastError();
    }
    if (a.nvec < 1 || a.nvec > kMaxFewVectors || (a.nvec > 1 && !gemv_bf16_takes_few(pattern, a))) return hipErrorInvalidValue;
    if (a.nvec > 1) {
        if (a.nvec <= 2) launch_few<2>(pattern, a, s);
        else if (a.nvec <= 4) launch_few<4>(pattern, a, s);
        else launch_few<8>(pattern, a, s);
        return hipGetLastError();
    }
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
