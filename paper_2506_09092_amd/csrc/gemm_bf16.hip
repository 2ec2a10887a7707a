// bf16 x bf16 -> fp32 GEMM for gfx950: C[M x N] = A[M x K] . B[K x N] with A
// row-major and B column-major, so both operands are contiguous along k (the
// same product as the paper's Task 2, at the reduced input precision that
// matrix cores are built for; accumulation and output stay fp32).
//
// This file holds the general-purpose kernel: any shape, any alignment, three
// tile sizes.  Large aligned problems go to the kernel in gemm_bf16_main.hip.
//
// One workgroup of 256 lanes (4 wavefronts, 2 x 2) owns a (64 T) x (64 T) tile
// of C, each wavefront T x T blocks of V_MFMA_F32_32X32X16_BF16: lane l
// supplies eight consecutive k (16 bytes) of row l % 32, k-offset 8 * (l / 32),
// for each operand -- one 16-byte LDS read per operand block and k-step.  Per
// K-tile of 64 (one 128-byte row per tile row, four k-steps) A[BM x 64] and
// B^T[BN x 64] are staged through registers into double-buffered LDS; staging
// through registers is what lets ragged edges be zero-filled lane by lane.
//
// LDS rows are 128 bytes with no padding; the 16-byte chunk c of row r is kept
// at chunk position c ^ ((r >> 1) & 7), so that the 16 rows that one group of
// lanes reads at one k-offset cover all 64 banks exactly once.
//
// The loop is an explicit schedule, fenced so the compiler keeps it: every
// MFMA of k-step kk is followed by its share of that k-step's other
// instructions -- the fragment reads of k-step kk+1, then LDS stores of the
// next K-tile (k-steps 0 and 1) or global loads of the one after (k-steps 2 and
// 3, each register reloaded only after it has been stored).  The one barrier
// per K-tile follows k-step 2: the last fragments of this stage are in
// registers by then and the next stage is completely written.
#include <type_traits>

#include "common.hpp"

namespace fsrgemm {
namespace {

constexpr int kThreads = 256;
constexpr int kBK = 64;                 // bf16 elements per K-tile: one 128-byte row
constexpr int kRowBytes = kBK * 2;

template <int MODE>
__device__ __forceinline__ u32x4 load8(const uint16_t *__restrict__ p, bool row_ok, int col, int col_limit)
{
    // p points at element (row, col); the vector covers col .. col+7 of that row.
    if constexpr (MODE == kFast) {
        return *reinterpret_cast<const u32x4 *>(p);
    } else {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (!row_ok) return v;
        if constexpr (MODE == kVecPred) {
            if (col + 7 < col_limit) return *reinterpret_cast<const u32x4 *>(p);
        }
#pragma unroll
        for (int t = 0; t < 8; ++t)
            if (col + t < col_limit) v[t / 2] |= (uint32_t)p[t] << (16 * (t % 2));
        return v;
    }
}

template <int T, int MIN_WAVES, int MODE>
__global__ __launch_bounds__(kThreads, MIN_WAVES) void gemm_bf16_kernel(GemmArgs g, int tiles_m, int tiles_n)
{
    constexpr int BM = 64 * T, BN = 64 * T;
    constexpr int TILE_B = BM * kRowBytes;          // bytes of one operand tile
    constexpr int STAGE_B = 2 * TILE_B;             // A + B
    constexpr int NV = BM / 32;                     // 16-byte vectors per lane per operand and K-tile
    constexpr int NG = 2 * NV;                      // ... of both operands
    constexpr int NR = 2 * T;                       // fragment reads per k-step
    constexpr int NMF = T * T;                      // MFMAs per k-step
    constexpr int NC = NR + NG / 2;                 // companion instructions per k-step
    constexpr int PER_SLOT = (NC + NMF - 1) / NMF;

    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const uint16_t *__restrict__ A = static_cast<const uint16_t *>(g.A);
    const uint16_t *__restrict__ B = static_cast<const uint16_t *>(g.B);
    float *__restrict__ C = g.C;
    const int M = g.M, N = g.N, K = g.K;
    int tile_m, tile_n;
    tile_coords(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave >> 1) * 32 * T, wn0 = (wave & 1) * 32 * T;
    const int li = lane & 31, lh = lane >> 5;
    const int nk = (K + kBK - 1) / kBK;

    if (nk == 0) {      // K == 0: every entry is an empty sum
        for (int e = tid; e < BM * BN; e += kThreads) {
            const int row = m0 + e / BN, col = n0 + e % BN;
            if (row < M && col < N) C[(int64_t)row * g.ldc + col] = 0.f;
        }
        return;
    }

    // Global side: per pass s the workgroup fetches 32 rows; lane covers row (tid >> 3) + 32 s, chunk tid & 7.
    const int grow = tid >> 3, gchunk = tid & 7;
    const uint16_t *a_ptr = A + (int64_t)(m0 + grow) * g.lda + gchunk * 8;
    const uint16_t *b_ptr = B + (int64_t)(n0 + grow) * g.ldb + gchunk * 8;
    const int64_t a_step = 32 * g.lda, b_step = 32 * g.ldb;
    u32x4 rg[NG];       // idx < NV: A pass idx; else B pass idx - NV
    auto gload = [&](int idx, int t) {      // K-tiles past the end are clamped: loaded again, never consumed
        const int k0 = (t < nk ? t : nk - 1) * kBK;
        if (idx < NV) rg[idx] = load8<MODE>(a_ptr + idx * a_step + k0, m0 + grow + 32 * idx < M, k0 + gchunk * 8, K);
        else rg[idx] = load8<MODE>(b_ptr + (idx - NV) * b_step + k0, n0 + grow + 32 * (idx - NV) < N, k0 + gchunk * 8, K);
    };
    const int w_off = grow * kRowBytes + ((gchunk ^ ((grow >> 1) & 7)) * 16);
    auto lwrite = [&](int stage, int idx) {
        char *p = smem + stage * STAGE_B + w_off + (idx < NV ? idx * 32 * kRowBytes : TILE_B + (idx - NV) * 32 * kRowBytes);
        *reinterpret_cast<u32x4 *>(p) = rg[idx];
    };
    // Fragment reads: block row li of the wavefront's A (or B) rows, k-chunk 2 kk + lh.
    const int ra0 = (wm0 + li) * kRowBytes, rb0 = TILE_B + (wn0 + li) * kRowBytes;
    const int rsw = (li >> 1) & 7;
    bf16x8 fa[2][T], fb[2][T];
    auto lread = [&](int stage, int kk, int fi, int idx) {    // idx < T: A block idx; else B block idx - T
        const int pos = ((2 * kk + lh) ^ rsw) * 16;
        const char *s = smem + stage * STAGE_B + pos;
        if (idx < T) fa[fi][idx] = *reinterpret_cast<const bf16x8 *>(s + ra0 + idx * 32 * kRowBytes);
        else fb[fi][idx - T] = *reinterpret_cast<const bf16x8 *>(s + rb0 + (idx - T) * 32 * kRowBytes);
    };

    f32x16 acc[T][T];
#pragma unroll
    for (int i = 0; i < T; ++i)
#pragma unroll
        for (int j = 0; j < T; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // K-tile t of parity P reads stage X = P; K-tile t+1 (in rg) is stored to Y = 1-P during k-steps 0 and 1,
    // rg is refilled with K-tile t+2 during k-steps 2 and 3.
    auto k_tile = [&](auto parity, int t) {
        constexpr int P = decltype(parity)::value;
        constexpr int X = P, Y = 1 - P;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int fc = kk & 1, fn = fc ^ 1;
#pragma unroll
            for (int m = 0; m < NMF; ++m) {
                acc[m / T][m % T] =
                    __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[fc][m / T], fb[fc][m % T], acc[m / T][m % T], 0, 0, 0);
#pragma unroll
                for (int c = m * PER_SLOT; c < (m + 1) * PER_SLOT && c < NC; ++c) {
                    if (c < NR) {
                        if (kk < 3) lread(X, kk + 1, fn, c); else lread(Y, 0, fn, c);
                    } else {
                        const int h = c - NR;       // 0 .. NG/2 - 1
                        if (kk == 0) lwrite(Y, h);
                        else if (kk == 1) lwrite(Y, NG / 2 + h);
                        else if (kk == 2) gload(h, t + 2);
                        else gload(NG / 2 + h, t + 2);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (kk == 2) {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // Prologue: K-tile 0 through the registers into stage 0, K-tile 1 into the registers, first fragments.
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

    // Register r of a 32x32 block holds row (r/4)*8 + 4*(lane/32) + r%4, column lane%32.
#pragma unroll
    for (int i = 0; i < T; ++i)
#pragma unroll
        for (int j = 0; j < T; ++j) {
            const int col = n0 + wn0 + j * 32 + li;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm0 + i * 32 + (r / 4) * 8 + lh * 4 + (r % 4);
                if (MODE == kFast || (row < M && col < N)) C[(int64_t)row * g.ldc + col] = acc[i][j][r];
            }
        }
}

template <int T, int MIN_WAVES, int MODE>
hipError_t launch_one(const GemmArgs &a, hipStream_t s)
{
    constexpr int BM = 64 * T;
    constexpr int lds = 2 * 2 * BM * kRowBytes;
    auto kern = gemm_bf16_kernel<T, MIN_WAVES, MODE>;
    static std::atomic<uint64_t> configured{0};
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds, configured);
    if (e != hipSuccess) return e;
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BM - 1) / BM;
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(kThreads), lds, s, a, tiles_m, tiles_n);
    return hipGetLastError();
}

template <int T, int MIN_WAVES>
hipError_t launch_cfg(int mode, const GemmArgs &a, hipStream_t s)
{
    switch (mode) {
    case kFast: return launch_one<T, MIN_WAVES, kFast>(a, s);
    case kVecPred: return launch_one<T, MIN_WAVES, kVecPred>(a, s);
    default: return launch_one<T, MIN_WAVES, kScalar>(a, s);
    }
}

}  // namespace

// <T, minimum wavefronts per SIMD, load mode>: tile (64 T) x (64 T); as a profiler trace prints the kernel
const char *bf16_kernel_name(int cfg, int mode)
{
    static const char *names[3][3] = {
        {"gemm_bf16_kernel<4, 1, 0>", "gemm_bf16_kernel<4, 1, 1>", "gemm_bf16_kernel<4, 1, 2>"},
        {"gemm_bf16_kernel<2, 2, 0>", "gemm_bf16_kernel<2, 2, 1>", "gemm_bf16_kernel<2, 2, 2>"},
        {"gemm_bf16_kernel<1, 4, 0>", "gemm_bf16_kernel<1, 4, 1>", "gemm_bf16_kernel<1, 4, 2>"},
    };
    return cfg == kBf16_Main ? bf16_main_kernel_name() : names[cfg - 1][mode];
}

hipError_t launch_bf16(int cfg, int mode, const GemmArgs &a, hipStream_t s)
{
    switch (cfg) {
    case kBf16_Main: return launch_bf16_main(a, s);
    case kBf16_256x256: return launch_cfg<4, 1>(mode, a, s);
    case kBf16_128x128: return launch_cfg<2, 2>(mode, a, s);
    default: return launch_cfg<1, 4>(mode, a, s);
    }
}

}  // namespace fsrgemm
