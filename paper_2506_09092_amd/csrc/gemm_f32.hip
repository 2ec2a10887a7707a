// fp32 GEMM for gfx950: C[M x N] = A[M x K] . B[K x N], all row-major
// (the paper's Task 2 definition: a 32-bit floating point matrix product).
//
// One workgroup of 256 lanes (4 wavefronts in a 2 x 2 grid) owns a
// (64 TM) x (64 TN) tile of C, each wavefront a (32 TM) x (32 TN) part of it as
// TM x TN blocks of V_MFMA_F32_32X32X2_F32.  Per K-tile of 16 the workgroup
// stages A[BM x 16] and B[16 x BN] through registers into a double-buffered
// LDS region.
//
// Operand mapping.  The 32x32x2 MFMA takes, per lane l, one A value
// A[l % 32][l / 32] and one B value B[l / 32][l % 32].  A is contiguous along
// k in memory and in LDS, so a lane fetches four consecutive k with a single
// 16-byte LDS read.  To make that useful the eight k of a chunk are assigned to
// MFMA steps in permuted order: lanes 0-31 hold k = 0..3, lanes 32-63 hold
// k = 4..7, and step t contracts the pair {t, 4 + t}.  B is read to match
// (row 4h + t for half h).  The sum over k is unchanged; only its order is.
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
// loads (any alignment).  Ragged modes also mask the stores.
#include <type_traits>

#include "common.hpp"

namespace fsrgemm {
namespace {

constexpr int kThreads = 256;
constexpr int kBK = 16;
constexpr int kPadA = 4;    // As row = 20 floats: 16-byte aligned; 16 consecutive rows hit distinct bank quads
constexpr int kPadB = 8;    // Bs row = BN + 8 floats: rows 4 apart land 32 banks apart

template <int MODE>
__device__ __forceinline__ f32x4 load4(const float *__restrict__ p, bool row_ok, int col, int col_limit)
{
    // p points at element (row, col); the vector covers col .. col+3 of that row.
    if constexpr (MODE == kFast) {
        return *reinterpret_cast<const f32x4 *>(p);
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

template <int TM, int TN, int MIN_WAVES, int MODE>
__global__ __launch_bounds__(kThreads, MIN_WAVES) void gemm_f32_kernel(GemmArgs g, int tiles_m, int tiles_n)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int LDA_S = kBK + kPadA, LDB_S = BN + kPadB;
    constexpr int A_ST = BM * LDA_S, B_ST = kBK * LDB_S;    // floats per LDS stage
    constexpr int NA = BM / 64, NB = BN / 64, NG = NA + NB;   // 16-byte vectors per lane per K-tile
    constexpr int NR = TM + 4 * TN;                           // fragment reads per 8-k chunk
    constexpr int NMF = 4 * TM * TN;                          // MFMAs per chunk
    constexpr int NC = NR + NG;                               // companion instructions per chunk
    constexpr int PER_SLOT = (NC + NMF - 1) / NMF;            // 1 for the large tiles, 2 for 64 x 64

    __shared__ __attribute__((aligned(16))) float As[2 * A_ST];
    __shared__ __attribute__((aligned(16))) float Bs[2 * B_ST];

    const float *__restrict__ A = static_cast<const float *>(g.A);
    const float *__restrict__ B = static_cast<const float *>(g.B);
    float *__restrict__ C = g.C;
    const int M = g.M, N = g.N, K = g.K;
    int tile_m, tile_n;
    tile_coords(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave >> 1) * 32 * TM, wn0 = (wave & 1) * 32 * TN;
    const int li = lane & 31, lh = lane >> 5;
    const int nk = (K + kBK - 1) / kBK;

    if (nk == 0) {      // K == 0: every entry is an empty sum
        for (int e = tid; e < BM * BN; e += kThreads) {
            const int row = m0 + e / BN, col = n0 + e % BN;
            if (row < M && col < N) C[(int64_t)row * g.ldc + col] = 0.f;
        }
        return;
    }

    // A tile: lane -> row (tid >> 2) + 64 s, columns 4 (tid & 3) ..; B tile: vector e = tid + 256 s -> row e / (BN/4)
    const int a_row = tid >> 2, a_col = (tid & 3) * 4;
    const float *a_ptr = A + (int64_t)(m0 + a_row) * g.lda + a_col;
    const int64_t a_step = 64 * g.lda;
    f32x4 rg[NG];
    auto gload = [&](int idx, int t) {      // K-tiles past the end are clamped: loaded again, never consumed
        const int k0 = (t < nk ? t : nk - 1) * kBK;
        if (idx < NA) {
            rg[idx] = load4<MODE>(a_ptr + idx * a_step + k0, m0 + a_row + 64 * idx < M, k0 + a_col, K);
        } else {
            const int e = tid + kThreads * (idx - NA);
            const int kr = k0 + e / (BN / 4), nc = n0 + (e % (BN / 4)) * 4;
            rg[idx] = load4<MODE>(B + (int64_t)kr * g.ldb + nc, kr < K, nc, N);
        }
    };
    const int aw = a_row * LDA_S + a_col;
    auto lwrite = [&](int stage, int idx) {
        if (idx < NA) {
            *reinterpret_cast<f32x4 *>(&As[stage * A_ST + aw + idx * 64 * LDA_S]) = rg[idx];
        } else {
            const int e = tid + kThreads * (idx - NA);
            *reinterpret_cast<f32x4 *>(&Bs[stage * B_ST + (e / (BN / 4)) * LDB_S + (e % (BN / 4)) * 4]) = rg[idx];
        }
    };
    const int ar = (wm0 + li) * LDA_S + 4 * lh, br = (4 * lh) * LDB_S + wn0 + li;
    f32x4 fa[2][TM];
    float fb[2][TN][4];
    auto lread = [&](int stage, int kk, int fi, int idx) {    // idx < TM: A block idx; then B, step-major
        if (idx < TM) {
            fa[fi][idx] = *reinterpret_cast<const f32x4 *>(&As[stage * A_ST + ar + idx * 32 * LDA_S + kk * 8]);
        } else {
            const int q = idx - TM, j = q % TN, t = q / TN;
            fb[fi][j][t] = Bs[stage * B_ST + br + (kk * 8 + t) * LDB_S + j * 32];
        }
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
    auto k_tile = [&](auto parity, int t) {
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
                        if (kk == 0) lwrite(Y, c - NR); else gload(c - NR, t + 2);
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

#pragma unroll
    for (int idx = 0; idx < NG; ++idx) gload(idx, 0);
#pragma unroll
    for (int idx = 0; idx < NG; ++idx) lwrite(0, idx);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int idx = 0; idx < NG; ++idx) gload(idx, 1);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int idx = 0; idx < NR; ++idx) lread(0, 0, 0, idx);
    __builtin_amdgcn_sched_barrier(0);

    int t = 0;
    for (; t + 1 < nk; t += 2) {
        k_tile(std::integral_constant<int, 0>{}, t);
        k_tile(std::integral_constant<int, 1>{}, t + 1);
    }
    if (t < nk) k_tile(std::integral_constant<int, 0>{}, t);

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

template <int TM, int TN, int MIN_WAVES>
hipError_t launch_cfg(int mode, const GemmArgs &a, hipStream_t s)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(kThreads);
    switch (mode) {
    case kFast: hipLaunchKernelGGL((gemm_f32_kernel<TM, TN, MIN_WAVES, kFast>), grid, block, 0, s, a, tiles_m, tiles_n); break;
    case kVecPred: hipLaunchKernelGGL((gemm_f32_kernel<TM, TN, MIN_WAVES, kVecPred>), grid, block, 0, s, a, tiles_m, tiles_n); break;
    default: hipLaunchKernelGGL((gemm_f32_kernel<TM, TN, MIN_WAVES, kScalar>), grid, block, 0, s, a, tiles_m, tiles_n); break;
    }
    return hipGetLastError();
}

}  // namespace

// <TM, TN, minimum wavefronts per SIMD, load mode>, as a profiler trace prints the kernel
const char *f32_kernel_name(int cfg, int mode)
{
    static const char *names[kF32ConfigCount][3] = {
        {"gemm_f32_kernel<4, 2, 2, 0>", "gemm_f32_kernel<4, 2, 2, 1>", "gemm_f32_kernel<4, 2, 2, 2>"},
        {"gemm_f32_kernel<2, 2, 3, 0>", "gemm_f32_kernel<2, 2, 3, 1>", "gemm_f32_kernel<2, 2, 3, 2>"},
        {"gemm_f32_kernel<1, 1, 4, 0>", "gemm_f32_kernel<1, 1, 4, 1>", "gemm_f32_kernel<1, 1, 4, 2>"},
    };
    return names[cfg][mode];
}

hipError_t launch_f32(int cfg, int mode, const GemmArgs &a, hipStream_t s)
{
    switch (cfg) {
    case kF32_256x128: return launch_cfg<4, 2, 2>(mode, a, s);
    case kF32_128x128: return launch_cfg<2, 2, 3>(mode, a, s);
    default: return launch_cfg<1, 1, 4>(mode, a, s);
    }
}

}  // namespace fsrgemm
