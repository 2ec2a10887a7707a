// fp32 GEMM for gfx950: C[M x N] = A[M x K] . B[K x N], C row-major, each
// operand stored row-major or transposed (the paper's Task 2 definition: a
// 32-bit floating point matrix product; the paper fixes no storage order for it).
//
// One workgroup of 256 lanes (4 wavefronts in a 2 x 2 grid) owns a
// (64 TM) x (64 TN) tile of C, each wavefront a (32 TM) x (32 TN) part of it as
// TM x TN blocks of V_MFMA_F32_32X32X2_F32.  Per K-tile of 16 the workgroup
// stages A[BM x 16] and B[16 x BN] through registers into a double-buffered
// LDS region.
//
// Operand layouts.  What matters to the kernel is which index of an operand
// tile is contiguous in memory: k (a row-major A, a transposed B) or the m / n
// index (a transposed A, a row-major B).  LDS keeps the memory order, so global
// loads and LDS stores are 16-byte vectors either way.
//
// Operand mapping.  The 32x32x2 MFMA takes, per lane l, one A value
// A[l % 32][l / 32] and one B value B[l / 32][l % 32].  An operand that is
// contiguous along k lets a lane fetch four consecutive k with a single 16-byte
// LDS read.  To make that useful the eight k of a chunk are assigned to MFMA
// steps in permuted order: lanes 0-31 hold k = 0..3, lanes 32-63 hold
// k = 4..7, and step t contracts the pair {t, 4 + t}.  An operand contiguous
// along m / n is read to match, one value per step (row 4h + t for half h).
// The sum over k is unchanged; only its order is.
//
// The loop is an explicit schedule: every MFMA is followed by its share of the
// other instructions of the chunk -- LDS fragment reads for the next 8-k chunk,
// LDS stores of the next K-tile or global loads of the one after -- and each
// group is fenced so the compiler keeps that order.  Operands are therefore in
// registers a full chunk before they are used, and the single barrier per
// K-tile sits between the two chunks, where nothing is waiting on it.
//
// Three load modes share the code: unchecked 16-byte vectors (aligned problems
// that are a whole number of tiles with K a multiple of 16), vectors with
// element-wise zero-filled edges (aligned, ragged), element-wise predicated
// loads (any alignment).  Ragged modes also mask the stores.  In the second
// and third mode a workgroup whose tile lies inside the matrix runs its whole
// K-tiles through unchecked loads (16-byte loads from merely element-aligned
// addresses in the third) and only the ragged end of K through the checked
// ones, so a ragged or unaligned problem pays for its edges only at its edges.
#include <stdio.h>

#include <type_traits>

#include "launchers.hpp"

namespace fsrgemm {
namespace {

constexpr int kThreads = 256;
constexpr int kBK = 16;
constexpr int kPadA = 4;    // As row = 20 floats: 16-byte aligned; 16 consecutive rows hit distinct bank quads
constexpr int64_t kMaxLdUnchecked = kF32MaxLdUnchecked;
constexpr int kPadB = 8;    // Bs row = BN + 8 floats: rows 4 apart land 32 banks apart

template <int MODE>
__device__ __forceinline__ f32x4 load4(const float *__restrict__ p, bool row_ok, int col, int col_limit)
{
    // p points at element (row, col); the vector covers col .. col+3 of that row.
    if constexpr (MODE == kFast) {
        return *reinterpret_cast<const f32x4 *>(p);
    } else if constexpr (MODE == kUnalignedVec) {
        f32x4 v;
        __builtin_memcpy(&v, p, sizeof v);
        return v;
    } else {
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (!row_ok) return v;
        if constexpr (MODE == kVecPred) {
            if (col + 3 < col_limit) return *reinterpret_cast<const f32x4 *>(p);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if (col + t < col_limit) v[t] = p[t];
        return v;
    }
}

// One operand tile of EXT rows (m or n) by kBK columns (k), in either storage order.
//   kKContig : element (r, k) at base[r * ld + k]; LDS rows of kBK + kPadA floats, one per r
//   kMnContig: element (r, k) at base[k * ld + r]; LDS rows of EXT + kPadB floats, one per k
// Either way a lane moves EXT / 64 16-byte vectors per K-tile.
template <int EXT, int LAY>
struct Operand {
    static constexpr int kRow = LAY == kKContig ? kBK + kPadA : EXT + kPadB;              // LDS row stride, floats
    static constexpr int kStage = LAY == kKContig ? EXT * (kBK + kPadA) : kBK * (EXT + kPadB);   // floats per stage
    static constexpr int kVectors = EXT / 64;
    static constexpr int kReads = LAY == kKContig ? 1 : 4;      // fragment reads per 32-row block and 8-k chunk

    // vector s of this lane: tile row / k column it starts at (kKContig: 4 consecutive k; kMnContig: 4 consecutive rows)
    static __device__ __forceinline__ void where(int tid, int s, int &r, int &k)
    {
        if constexpr (LAY == kKContig) {
            r = (tid >> 2) + 64 * s;
            k = (tid & 3) * 4;
        } else {
            const int e = tid + kThreads * s;
            k = e / (EXT / 4);
            r = (e % (EXT / 4)) * 4;
        }
    }
    template <int MODE>
    static __device__ __forceinline__ f32x4 gload(const float *__restrict__ base, int64_t ld, int r0, int rows, int k0,
                                                  int K, int tid, int s)
    {
        int r, k;
        where(tid, s, r, k);
        if constexpr (LAY == kKContig)
            return load4<MODE>(base + (int64_t)(r0 + r) * ld + k0 + k, r0 + r < rows, k0 + k, K);
        else
            return load4<MODE>(base + (int64_t)(k0 + k) * ld + r0 + r, k0 + k < K, r0 + r, rows);
    }
    // Unchecked loads take their address as a wavefront-uniform 64-bit base (the tile's origin, the K position and
    // vector s: scalar registers, computed by the scalar unit) plus a 32-bit byte offset per lane that is the same for
    // every vector and K-tile.  In that form a load reads one address register per lane instead of two and needs no
    // vector arithmetic; with 64-bit lane addresses each load held the matrix pipe up for some 40 cycles.
    // Needs ld < 2^24 (kMaxLdUnchecked): the offset reaches (63 ld + 15) * 4 bytes.
    static __device__ __forceinline__ uint32_t lane_offset(int tid, int64_t ld)
    {
        if constexpr (LAY == kKContig) return (uint32_t)(((tid >> 2) * ld + (tid & 3) * 4) * 4);
        else return (uint32_t)(((tid / (EXT / 4)) * ld + (tid % (EXT / 4)) * 4) * 4);
    }
    // the uniform part for vector s of the K-tile that starts at k0, and what one K-tile further adds to it (bytes)
    static __device__ __forceinline__ const char *vector_base(const float *__restrict__ base, int64_t ld, int r0, int k0, int s)
    {
        static_assert(256 % (EXT / 4) == 0, "vector s of a lane must start a whole number of k-rows behind vector 0");
        if constexpr (LAY == kKContig) return reinterpret_cast<const char *>(base + (int64_t)(r0 + 64 * s) * ld + k0);
        else return reinterpret_cast<const char *>(base + (int64_t)(k0 + s * (1024 / EXT)) * ld + r0);
    }
    static __device__ __forceinline__ int64_t k_tile_step(int64_t ld) { return LAY == kKContig ? kBK * 4 : kBK * 4 * ld; }
    template <int MODE>
    static __device__ __forceinline__ f32x4 gload_unchecked(const char *u, uint32_t lane_off)
    {
        static_assert(MODE == kFast || MODE == kUnalignedVec, "checked loads go through gload");
        // opaque to the optimiser, so that base and offset reach instruction selection as they are written here
        // (it would otherwise fold the offset into a 64-bit address per lane outside the loop)
        asm volatile("" : "+s"(u), "+v"(lane_off));
        const __attribute__((address_space(1))) char *p = (const __attribute__((address_space(1))) char *)u + lane_off;
        if constexpr (MODE == kFast) {
            return *reinterpret_cast<const __attribute__((address_space(1))) f32x4 *>(p);
        } else {
            typedef f32x4 f32x4_elem_aligned __attribute__((aligned(4)));
            return *reinterpret_cast<const __attribute__((address_space(1))) f32x4_elem_aligned *>(p);
        }
    }
    static __device__ __forceinline__ int lds_store_at(int tid, int s)
    {
        int r, k;
        where(tid, s, r, k);
        return LAY == kKContig ? r * kRow + k : k * kRow + r;
    }
    // fragment read `q` of block `blk` for chunk kk; w = wavefront's first row + lane % 32, h = lane / 32
    static __device__ __forceinline__ void fragment(const float *stage, int w, int h, int blk, int kk, int q, f32x4 &f)
    {
        if constexpr (LAY == kKContig)
            f = *reinterpret_cast<const f32x4 *>(&stage[(w + 32 * blk) * kRow + 4 * h + kk * 8]);
        else
            f[q] = stage[(kk * 8 + 4 * h + q) * kRow + w + 32 * blk];
    }
};

template <int TM, int TN, int MIN_WAVES, int MODE, int ALAY, int BLAY>
__global__ __launch_bounds__(kThreads, MIN_WAVES) void gemm_f32_kernel(GemmArgs g, int tiles_m, int tiles_n)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    using OpA = Operand<BM, ALAY>;
    using OpB = Operand<BN, BLAY>;
    constexpr int A_ST = OpA::kStage, B_ST = OpB::kStage;     // floats per LDS stage
    constexpr int NA = OpA::kVectors, NB = OpB::kVectors, NG = NA + NB;   // 16-byte vectors per lane per K-tile
    constexpr int NRA = OpA::kReads * TM, NR = NRA + OpB::kReads * TN;    // fragment reads per 8-k chunk
    constexpr int NMF = 4 * TM * TN;                          // MFMAs per chunk
    constexpr int NC = NR + NG;                               // companion instructions per chunk
    constexpr int PER_SLOT = (NC + NMF - 1) / NMF;            // 1 for the large row-major tiles, up to 3 for 64 x 64

    __shared__ __attribute__((aligned(16))) float As[2 * A_ST];
    __shared__ __attribute__((aligned(16))) float Bs[2 * B_ST];

    const float *__restrict__ A = static_cast<const float *>(g.A);
    const float *__restrict__ B = static_cast<const float *>(g.B);
    const int M = g.M, N = g.N, K = g.K;
    // Split-K: workgroup ids beyond the first tiles_m * tiles_n belong to further K slices.  Slice s takes
    // K-tiles [s * per, (s + 1) * per) of the whole range and writes its partial product to the s-th M x N
    // block behind g.C (a workspace then, tightly packed: the launcher sets ldc = N).
    const int tiles = tiles_m * tiles_n;
    const int slice = g.k_slices > 1 ? (int)blockIdx.x / tiles : 0;
    const int nk_all = (K + kBK - 1) / kBK;
    const int per = (nk_all + g.k_slices - 1) / g.k_slices;
    const int t0 = slice * per;                                     // first K-tile of this slice
    const int nk = max(0, min(per, nk_all - t0));
    float *__restrict__ C = g.C + (int64_t)slice * g.slice_stride;
    int tile_m, tile_n;
    tile_coords((int)blockIdx.x - slice * tiles, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_origin(tile_m, BM, M), n0 = tile_origin(tile_n, BN, N);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave >> 1) * 32 * TM, wn0 = (wave & 1) * 32 * TN;
    const int li = lane & 31, lh = lane >> 5;

    if (nk == 0) {      // K == 0 (or a slice past the end of K): every entry is an empty sum
        for (int e = tid; e < BM * BN; e += kThreads) {
            const int row = m0 + e / BN, col = n0 + e % BN;
            if (row < M && col < N) C[(int64_t)row * g.ldc + col] = 0.f;
        }
        return;
    }

    // A workgroup whose tile lies inside the matrix needs no check on whole K-tiles even when the problem as a
    // whole is ragged: `unchecked` counts the leading K-tiles it may load like the unchecked mode does.
    const bool offsets_fit = g.lda < kMaxLdUnchecked && g.ldb < kMaxLdUnchecked;     // the unchecked mode is only launched if so
    const int unchecked = MODE == kFast ? nk : (offsets_fit && m0 + BM <= M && n0 + BN <= N) ? max(0, min(nk, K / kBK - t0)) : 0;
    const uint32_t a_lane = OpA::lane_offset(tid, g.lda), b_lane = OpB::lane_offset(tid, g.ldb);
    // Uniform bases of the unchecked loads, one per vector, for the K-tile such a load fetches next: they walk K one
    // tile per use (unchecked loads fetch K-tiles in order, starting with the slice's first) and stop at the last.
    const char *ua[NA], *ub[NB];
#pragma unroll
    for (int s = 0; s < NA; ++s) ua[s] = OpA::vector_base(A, g.lda, m0, t0 * kBK, s);
#pragma unroll
    for (int s = 0; s < NB; ++s) ub[s] = OpB::vector_base(B, g.ldb, n0, t0 * kBK, s);
    const int64_t a_step = OpA::k_tile_step(g.lda), b_step = OpB::k_tile_step(g.ldb);
    f32x4 rg[NG];
    auto gload = [&](auto load_mode, int idx, int t) {      // K-tiles past the end are clamped: loaded again, never consumed
        constexpr int LM = decltype(load_mode)::value;
        const int k0 = (t0 + (t < nk ? t : nk - 1)) * kBK;
        // The smallest tile keeps an address per lane for its unchecked loads too: it has a single accumulator block,
        // so its MFMAs form one dependent chain and a workgroup alone is bound by load latency; with few workgroups
        // per compute unit the scalar-base form (whose base is computed on the wavefront's own instruction stream)
        // measured 7-9 % slower there (1024 x 2048 x 4096, 3072^2), though 8 % faster with many (5120^2).
        if constexpr ((LM == kFast || LM == kUnalignedVec) && TM * TN > 1) {
            const bool more = t + 1 < nk;
            if (idx < NA) {
                rg[idx] = OpA::template gload_unchecked<LM>(ua[idx], a_lane);
                ua[idx] += more ? a_step : 0;
            } else {
                rg[idx] = OpB::template gload_unchecked<LM>(ub[idx - NA], b_lane);
                ub[idx - NA] += more ? b_step : 0;
            }
        } else {
            if (idx < NA) rg[idx] = OpA::template gload<LM>(A, g.lda, m0, M, k0, K, tid, idx);
            else rg[idx] = OpB::template gload<LM>(B, g.ldb, n0, N, k0, K, tid, idx - NA);
        }
    };
    using Checked = std::integral_constant<int, MODE>;
    using Unchecked = std::integral_constant<int, MODE == kScalar ? kUnalignedVec : kFast>;
    auto lwrite = [&](int stage, int idx) {
        if (idx < NA) *reinterpret_cast<f32x4 *>(&As[stage * A_ST + OpA::lds_store_at(tid, idx)]) = rg[idx];
        else *reinterpret_cast<f32x4 *>(&Bs[stage * B_ST + OpB::lds_store_at(tid, idx - NA)]) = rg[idx];
    };
    f32x4 fa[2][TM], fb[2][TN];     // component t of a fragment feeds MFMA step t of the chunk
    auto lread = [&](int stage, int kk, int fi, int idx) {    // A's reads first, then B's; block-minor
        if (idx < NRA) OpA::fragment(&As[stage * A_ST], wm0 + li, lh, idx % TM, kk, idx / TM, fa[fi][idx % TM]);
        else OpB::fragment(&Bs[stage * B_ST], wn0 + li, lh, (idx - NRA) % TN, kk, (idx - NRA) / TN, fb[fi][(idx - NRA) % TN]);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // K-tile t of parity P reads stage P.  Chunk 0: fragments of chunk 1, then the staged K-tile t+1 goes to
    // stage 1-P; barrier.  Chunk 1: fragments of K-tile t+1's chunk 0 from stage 1-P, then global loads of t+2.
    auto k_tile = [&](auto parity, auto load_mode, int t) {
        constexpr int P = decltype(parity)::value;
        constexpr int X = P, Y = 1 - P;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int fc = kk, fn = kk ^ 1;
#pragma unroll
            for (int m = 0; m < NMF; ++m) {
                const int tt = m / (TM * TN), i = (m / TN) % TM, j = m % TN;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[fc][i][tt], fb[fc][j][tt], acc[i][j], 0, 0, 0);
#pragma unroll
                for (int c = m * PER_SLOT; c < (m + 1) * PER_SLOT && c < NC; ++c) {
                    if (c < NR) {
                        if (kk == 0) lread(X, 1, fn, c); else lread(Y, 0, fn, c);
                    } else {
                        if (kk == 0) lwrite(Y, c - NR); else gload(load_mode, c - NR, t + 2);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (kk == 0) {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    if (MODE != kFast && unchecked >= 1) {
#pragma unroll
        for (int idx = 0; idx < NG; ++idx) gload(Unchecked{}, idx, 0);
    } else {
#pragma unroll
        for (int idx = 0; idx < NG; ++idx) gload(Checked{}, idx, 0);
    }
#pragma unroll
    for (int idx = 0; idx < NG; ++idx) lwrite(0, idx);
    __builtin_amdgcn_sched_barrier(0);
    if (MODE != kFast && unchecked >= 2) {
#pragma unroll
        for (int idx = 0; idx < NG; ++idx) gload(Unchecked{}, idx, 1);
    } else {
#pragma unroll
        for (int idx = 0; idx < NG; ++idx) gload(Checked{}, idx, 1);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int idx = 0; idx < NR; ++idx) lread(0, 0, 0, idx);
    __builtin_amdgcn_sched_barrier(0);

    int t = 0;
    if constexpr (MODE != kFast) {
        // K-tile t loads K-tile t + 2: this loop runs while t + 3 is still an unchecked K-tile
        for (; t + 3 < unchecked; t += 2) {
            k_tile(std::integral_constant<int, 0>{}, Unchecked{}, t);
            k_tile(std::integral_constant<int, 1>{}, Unchecked{}, t + 1);
        }
    }
    for (; t + 1 < nk; t += 2) {
        k_tile(std::integral_constant<int, 0>{}, Checked{}, t);
        k_tile(std::integral_constant<int, 1>{}, Checked{}, t + 1);
    }
    if (t < nk) k_tile(std::integral_constant<int, 0>{}, Checked{}, t);

    // Register r of a 32x32 block holds row (r/4)*8 + 4*(lane/32) + r%4, column lane%32: each store
    // instruction writes two 128-byte row segments.
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn0 + j * 32 + li;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm0 + i * 32 + (r / 4) * 8 + lh * 4 + (r % 4);
                if (MODE == kFast || (row < M && col < N)) C[(int64_t)row * g.ldc + col] = acc[i][j][r];
            }
        }
}

template <int TM, int TN, int MIN_WAVES, int ALAY, int BLAY>
hipError_t launch_lay(int mode, const GemmArgs &args, hipStream_t s)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    const GemmArgs &a = args;
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const dim3 grid((unsigned)(tiles_m * tiles_n * a.k_slices)), block(kThreads);
    switch (mode) {
    case kFast: hipLaunchKernelGGL((gemm_f32_kernel<TM, TN, MIN_WAVES, kFast, ALAY, BLAY>), grid, block, 0, s, a, tiles_m, tiles_n); break;
    case kVecPred: hipLaunchKernelGGL((gemm_f32_kernel<TM, TN, MIN_WAVES, kVecPred, ALAY, BLAY>), grid, block, 0, s, a, tiles_m, tiles_n); break;
    default: hipLaunchKernelGGL((gemm_f32_kernel<TM, TN, MIN_WAVES, kScalar, ALAY, BLAY>), grid, block, 0, s, a, tiles_m, tiles_n); break;
    }
    return hipGetLastError();
}

template <int TM, int TN, int MIN_WAVES>
hipError_t launch_cfg(int mode, int a_lay, int b_lay, const GemmArgs &a, hipStream_t s)
{
    if (a_lay == kKContig) {
        return b_lay == kMnContig ? launch_lay<TM, TN, MIN_WAVES, kKContig, kMnContig>(mode, a, s)
                                  : launch_lay<TM, TN, MIN_WAVES, kKContig, kKContig>(mode, a, s);
    }
    return b_lay == kMnContig ? launch_lay<TM, TN, MIN_WAVES, kMnContig, kMnContig>(mode, a, s)
                              : launch_lay<TM, TN, MIN_WAVES, kMnContig, kKContig>(mode, a, s);
}

}  // namespace

namespace {

// C[i][j] = ws[0][i][j] + ws[1][i][j] + ... in that order: the second half of a split-K product.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ ws, int slices, int64_t slice_stride,
                                                            float *__restrict__ C, int M, int N, int64_t ldc)
{
    const int64_t total = (int64_t)M * N;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        float sum = ws[e];
        for (int s = 1; s < slices; ++s) sum += ws[(int64_t)s * slice_stride + e];
        C[(e / N) * ldc + e % N] = sum;
    }
}

}  // namespace

const char *splitk_reduce_kernel_name() { return "splitk_reduce_kernel"; }

hipError_t launch_splitk_reduce(const float *ws, int slices, int64_t slice_stride, float *C, int M, int N, int64_t ldc,
                                hipStream_t s)
{
    const int64_t total = (int64_t)M * N;
    const unsigned blocks = (unsigned)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks), dim3(256), 0, s, ws, slices, slice_stride, C, M, N, ldc);
    return hipGetLastError();
}

// <TM, TN, minimum wavefronts per SIMD, load mode, A layout, B layout>, as a profiler trace prints the kernel
const char *f32_kernel_name(int cfg, int mode, int a_lay, int b_lay)
{
    struct Names {
        char text[kF32ConfigCount][3][2][2][40];
        Names()
        {
            static const char *shapes[kF32ConfigCount] = {"4, 2, 2", "2, 2, 3", "1, 1, 4"};
            for (int c = 0; c < kF32ConfigCount; ++c)
                for (int m = 0; m < 3; ++m)
                    for (int x = 0; x < 2; ++x)
                        for (int y = 0; y < 2; ++y)
                            snprintf(text[c][m][x][y], sizeof text[c][m][x][y], "gemm_f32_kernel<%s, %d, %d, %d>",
                                     shapes[c], m, x, y);
        }
    };
    static const Names names;
    return names.text[cfg][mode][a_lay][b_lay];
}

hipError_t launch_f32(int cfg, int mode, int a_lay, int b_lay, const GemmArgs &a, hipStream_t s)
{
    if (mode == kFast && (a.lda >= kMaxLdUnchecked || a.ldb >= kMaxLdUnchecked)) return hipErrorInvalidValue;
    switch (cfg) {
    case kF32_256x128: return launch_cfg<4, 2, 2>(mode, a_lay, b_lay, a, s);
    case kF32_128x128: return launch_cfg<2, 2, 3>(mode, a_lay, b_lay, a, s);
    default: return launch_cfg<1, 1, 4>(mode, a_lay, b_lay, a, s);
    }
}

}  // namespace fsrgemm
