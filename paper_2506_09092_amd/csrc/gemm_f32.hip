// fp32 GEMM for gfx950: C[M x N] = A[M x K] . B[K x N], all row-major
// (the paper's Task 2 definition: a 32-bit floating point matrix product).
//
// One workgroup of 256 lanes (4 wavefronts in a 2 x 2 grid) owns a BM x BN tile
// of C.  Per K-tile of BK = 16 it stages A[BM x BK] and B[BK x BN] through a
// double-buffered LDS region and contracts them with V_MFMA_F32_32X32X2_F32,
// every wavefront keeping (BM/2) x (BN/2) accumulators in registers.
//
// Operand mapping.  The 32x32x2 MFMA takes, per lane l, one A value
// A[l % 32][l / 32] and one B value B[l / 32][l % 32].  A is contiguous along
// k in memory and in LDS, so a lane fetches four consecutive k with a single
// 16-byte LDS read.  To make that useful the eight k of a chunk are assigned to
// MFMA steps in permuted order: lanes 0-31 hold k = 0..3, lanes 32-63 hold
// k = 4..7, and step t contracts the pair {t, 4 + t}.  B is read to match
// (row 4h + t for half h).  The sum over k is unchanged; only its order is.
//
// Two kernels share that mapping.  gemm_f32_kernel is the general one (any
// shape and alignment, three load modes).  gemm_f32_sched_kernel serves
// aligned, tile-multiple problems: its loop is an explicit schedule in which
// every MFMA is followed by at most one other instruction -- an LDS fragment
// read for the next 8-k chunk, an LDS store of the next K-tile or a global load
// of the one after -- so that operands are always in registers a full chunk
// before they are used, and the single barrier per K-tile sits between the two
// chunks, where nothing is waiting on it.
#include <type_traits>

#include "common.hpp"

namespace fsrgemm {
namespace {

constexpr int kThreads = 256;
constexpr int kBK = 16;
constexpr int kPadA = 4;    // As row = 20 floats: 16-byte aligned, 8 rows hit 8 distinct bank quads
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

template <int BM, int BN, int MODE>
__global__ __launch_bounds__(kThreads) void gemm_f32_kernel(GemmArgs g, int tiles_m, int tiles_n)
{
    constexpr int WM = BM / 2, WN = BN / 2;       // wavefront tile
    constexpr int TM = WM / 32, TN = WN / 32;     // 32x32 MFMA blocks per wavefront
    constexpr int LDA_S = kBK + kPadA;
    constexpr int LDB_S = BN + kPadB;
    constexpr int NA = BM * kBK / 4 / kThreads;   // 16-byte vectors of A per lane per K-tile
    constexpr int NB = kBK * BN / 4 / kThreads;
    static_assert(NA >= 1 && NB >= 1, "tile too small for 256 lanes");

    __shared__ __attribute__((aligned(16))) float As[2][BM * LDA_S];
    __shared__ __attribute__((aligned(16))) float Bs[2][kBK * LDB_S];

    const float *__restrict__ A = static_cast<const float *>(g.A);
    const float *__restrict__ B = static_cast<const float *>(g.B);
    const int M = g.M, N = g.N, K = g.K;

    int tile_m, tile_n;
    tile_coords(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid % kWave, wave = tid / kWave;
    const int wm0 = (wave / 2) * WM, wn0 = (wave % 2) * WN;
    const int li = lane % 32, lh = lane / 32;

    // Global -> register staging coordinates.
    int a_row[NA], a_col[NA], b_row[NB], b_col[NB];
    const float *a_ptr[NA];
    const float *b_ptr[NB];
#pragma unroll
    for (int s = 0; s < NA; ++s) {
        const int e = tid + s * kThreads;
        a_row[s] = e / (kBK / 4);
        a_col[s] = (e % (kBK / 4)) * 4;
        a_ptr[s] = A + (int64_t)(m0 + a_row[s]) * g.lda + a_col[s];
    }
#pragma unroll
    for (int s = 0; s < NB; ++s) {
        const int e = tid + s * kThreads;
        b_row[s] = e / (BN / 4);
        b_col[s] = (e % (BN / 4)) * 4;
        b_ptr[s] = B + (int64_t)b_row[s] * g.ldb + n0 + b_col[s];
    }

    f32x4 ra[NA], rb[NB];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int s = 0; s < NA; ++s)
            ra[s] = load4<MODE>(a_ptr[s] + k0, m0 + a_row[s] < M, k0 + a_col[s], K);
#pragma unroll
        for (int s = 0; s < NB; ++s)
            rb[s] = load4<MODE>(b_ptr[s] + (int64_t)k0 * g.ldb, k0 + b_row[s] < K, n0 + b_col[s], N);
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int s = 0; s < NA; ++s)
            *reinterpret_cast<f32x4 *>(&As[buf][a_row[s] * LDA_S + a_col[s]]) = ra[s];
#pragma unroll
        for (int s = 0; s < NB; ++s)
            *reinterpret_cast<f32x4 *>(&Bs[buf][b_row[s] * LDB_S + b_col[s]]) = rb[s];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = (K + kBK - 1) / kBK;
    if (nk > 0) {
        fetch(0);
        stash(0);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) fetch((kt + 1) * kBK);

        const float *as = &As[buf][(wm0 + li) * LDA_S + 4 * lh];
        const float *bs = &Bs[buf][(4 * lh) * LDB_S + wn0 + li];
#pragma unroll
        for (int kk = 0; kk < kBK / 8; ++kk) {
            f32x4 af[TM];
            float bf[TN][4];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const f32x4 *>(as + i * 32 * LDA_S + kk * 8);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int t = 0; t < 4; ++t) bf[j][t] = bs[(kk * 8 + t) * LDB_S + j * 32];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][t], bf[j][t], acc[i][j], 0, 0, 0);
        }

        if (more) stash(buf ^ 1);
        __syncthreads();
    }

    // Epilogue.  Register r of a 32x32 block holds row (r/4)*8 + 4*(lane/32) + r%4,
    // column lane%32: each store instruction writes two 128-byte row segments.
    float *__restrict__ C = g.C;
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

// Scheduled kernel: tile (64 TM) x (64 TN) x 16, wavefront tile (32 TM) x (32 TN).
// Requires M % (64 TM) == 0, N % (64 TN) == 0, K % 16 == 0, K >= 16, 16-byte
// aligned A and B with lda % 4 == 0 and ldb % 4 == 0.
template <int TM, int TN, int MIN_WAVES>
__global__ __launch_bounds__(kThreads, MIN_WAVES) void gemm_f32_sched_kernel(GemmArgs g, int tiles_m, int tiles_n)
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
    int tile_m, tile_n;
    tile_coords(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave >> 1) * 32 * TM, wn0 = (wave & 1) * 32 * TN;
    const int li = lane & 31, lh = lane >> 5;
    const int nk = g.K / kBK;

    // A tile: lane -> row (tid >> 2) + 64 s, columns 4 (tid & 3) ..; B tile: vector e = tid + 256 s -> row e / (BN/4)
    const float *a_ptr = A + (int64_t)(m0 + (tid >> 2)) * g.lda + (tid & 3) * 4;
    const int64_t a_step = 64 * g.lda;
    f32x4 rg[NG];
    auto gload = [&](int idx, int t) {      // K-tiles past the end are clamped: loaded, never consumed
        const int tc = t < nk ? t : nk - 1;
        if (idx < NA) {
            rg[idx] = *reinterpret_cast<const f32x4 *>(a_ptr + idx * a_step + tc * kBK);
        } else {
            const int e = tid + kThreads * (idx - NA);
            rg[idx] = *reinterpret_cast<const f32x4 *>(B + (int64_t)(tc * kBK + e / (BN / 4)) * g.ldb + n0 + (e % (BN / 4)) * 4);
        }
    };
    const int aw = (tid >> 2) * LDA_S + (tid & 3) * 4;
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

    float *__restrict__ C = g.C;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn0 + j * 32 + li;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm0 + i * 32 + (r / 4) * 8 + lh * 4 + (r % 4);
                C[(int64_t)row * g.ldc + col] = acc[i][j][r];
            }
        }
}

template <int TM, int TN, int MIN_WAVES>
hipError_t launch_sched(const GemmArgs &a, hipStream_t s)
{
    const int tiles_m = a.M / (64 * TM), tiles_n = a.N / (64 * TN);
    hipLaunchKernelGGL((gemm_f32_sched_kernel<TM, TN, MIN_WAVES>), dim3((unsigned)(tiles_m * tiles_n)), dim3(kThreads), 0, s,
                       a, tiles_m, tiles_n);
    return hipGetLastError();
}

template <int BM, int BN>
hipError_t launch_cfg(int mode, const GemmArgs &a, hipStream_t s)
{
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(kThreads);
    switch (mode) {
    case kFast: hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, kFast>), grid, block, 0, s, a, tiles_m, tiles_n); break;
    case kVecPred: hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, kVecPred>), grid, block, 0, s, a, tiles_m, tiles_n); break;
    default: hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, kScalar>), grid, block, 0, s, a, tiles_m, tiles_n); break;
    }
    return hipGetLastError();
}

}  // namespace

const char *f32_kernel_name(int cfg, int mode)
{
    static const char *names[2][3] = {
        {"gemm_f32_kernel<128, 128, 0>", "gemm_f32_kernel<128, 128, 1>", "gemm_f32_kernel<128, 128, 2>"},
        {"gemm_f32_kernel<64, 64, 0>", "gemm_f32_kernel<64, 64, 1>", "gemm_f32_kernel<64, 64, 2>"},
    };
    if (cfg == kF32_Sched256x128) return "gemm_f32_sched_kernel<4, 2, 2>";
    if (cfg == kF32_Sched128x128) return "gemm_f32_sched_kernel<2, 2, 3>";
    if (cfg == kF32_Sched64x64) return "gemm_f32_sched_kernel<1, 1, 4>";
    return names[cfg - kF32_128x128][mode];
}

hipError_t launch_f32(int cfg, int mode, const GemmArgs &a, hipStream_t s)
{
    switch (cfg) {
    case kF32_Sched256x128: return launch_sched<4, 2, 2>(a, s);
    case kF32_Sched128x128: return launch_sched<2, 2, 3>(a, s);
    case kF32_Sched64x64: return launch_sched<1, 1, 4>(a, s);
    case kF32_128x128: return launch_cfg<128, 128>(mode, a, s);
    default: return launch_cfg<64, 64>(mode, a, s);
    }
}

}  // namespace fsrgemm
