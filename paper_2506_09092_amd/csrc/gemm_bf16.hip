// bf16 x bf16 -> fp32 GEMM for gfx950: C[M x N] = A[M x K] . B[K x N] with A
// row-major and B column-major, so both operands are contiguous along k (the
// same product as the paper's Task 2, at the reduced input precision that
// matrix cores are built for; accumulation and output stay fp32).
//
// A workgroup owns a BM x BN tile of C.  Per K-tile of BK = 64 it stages
// A[BM x 64] and B^T[BN x 64] (128 bytes per row) through double-buffered LDS
// and contracts with V_MFMA_F32_32X32X16_BF16: lane l supplies eight
// consecutive k (16 bytes) of row l % 32, k-offset 8 * (l / 32), for each
// operand -- exactly one 16-byte LDS read per operand block.
//
// LDS rows are 128 bytes with no padding; the 16-byte chunk c of row r is kept
// at chunk position c ^ ((r >> 1) & 7), so that the 16 rows that one group of
// lanes reads at one k-offset cover all 64 banks exactly once.
//
// This file holds the general-purpose configurations (any shape, any
// alignment); large aligned problems go to the scheduled kernel in
// gemm_bf16_main.hip.
#include "common.hpp"

namespace fsrgemm {
namespace {

constexpr int kBK = 64;                 // bf16 elements per K-tile: one 128-byte row
constexpr int kChunks = kBK / 8;        // 16-byte chunks per row

__device__ __forceinline__ int swizzled(int row, int chunk) { return row * kBK + ((chunk ^ ((row >> 1) & 7)) * 8); }

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

template <int BM, int BN, int WAVES_M, int WAVES_N, int MODE>
__global__ __launch_bounds__(WAVES_M *WAVES_N *kWave) void gemm_bf16_kernel(GemmArgs g, int tiles_m, int tiles_n)
{
    constexpr int THREADS = WAVES_M * WAVES_N * kWave;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int NA = BM * kChunks / THREADS;      // 16-byte vectors of A per lane per K-tile
    constexpr int NB = BN * kChunks / THREADS;
    static_assert(NA >= 1 && NB >= 1 && TM >= 1 && TN >= 1, "bad tile configuration");

    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t *As = smem;                            // [2][BM * 64]
    uint16_t *Bs = smem + 2 * BM * kBK;             // [2][BN * 64]

    const uint16_t *__restrict__ A = static_cast<const uint16_t *>(g.A);
    const uint16_t *__restrict__ B = static_cast<const uint16_t *>(g.B);
    const int M = g.M, N = g.N, K = g.K;

    int tile_m, tile_n;
    tile_coords(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid % kWave, wave = tid / kWave;
    const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
    const int li = lane % 32, lh = lane / 32;

    int a_row[NA], b_row[NB];
    const int chunk = tid % kChunks;                // same chunk column for every vector of a lane
    const uint16_t *a_ptr[NA];
    const uint16_t *b_ptr[NB];
#pragma unroll
    for (int s = 0; s < NA; ++s) {
        a_row[s] = (tid + s * THREADS) / kChunks;
        a_ptr[s] = A + (int64_t)(m0 + a_row[s]) * g.lda + chunk * 8;
    }
#pragma unroll
    for (int s = 0; s < NB; ++s) {
        b_row[s] = (tid + s * THREADS) / kChunks;
        b_ptr[s] = B + (int64_t)(n0 + b_row[s]) * g.ldb + chunk * 8;
    }

    u32x4 ra[NA], rb[NB];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int s = 0; s < NA; ++s) ra[s] = load8<MODE>(a_ptr[s] + k0, m0 + a_row[s] < M, k0 + chunk * 8, K);
#pragma unroll
        for (int s = 0; s < NB; ++s) rb[s] = load8<MODE>(b_ptr[s] + k0, n0 + b_row[s] < N, k0 + chunk * 8, K);
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int s = 0; s < NA; ++s)
            *reinterpret_cast<u32x4 *>(&As[buf * BM * kBK + swizzled(a_row[s], chunk)]) = ra[s];
#pragma unroll
        for (int s = 0; s < NB; ++s)
            *reinterpret_cast<u32x4 *>(&Bs[buf * BN * kBK + swizzled(b_row[s], chunk)]) = rb[s];
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

        const uint16_t *as = As + buf * BM * kBK;
        const uint16_t *bs = Bs + buf * BN * kBK;
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            bf16x8 af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8 *>(as + swizzled(wm0 + i * 32 + li, 2 * kk + lh));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bf[j] = *reinterpret_cast<const bf16x8 *>(bs + swizzled(wn0 + j * 32 + li, 2 * kk + lh));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }

        if (more) stash(buf ^ 1);
        __syncthreads();
    }

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

template <int BM, int BN, int WAVES_M, int WAVES_N, int MODE>
hipError_t launch_one(const GemmArgs &a, hipStream_t s)
{
    constexpr int THREADS = WAVES_M * WAVES_N * kWave;
    constexpr size_t lds = 2ull * (BM + BN) * kBK * sizeof(uint16_t);
    auto kern = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, MODE>;
    static bool configured = false;     // raising the dynamic-LDS limit is idempotent, so a race here is benign
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(THREADS), lds, s, a, tiles_m, tiles_n);
    return hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch_cfg(int mode, const GemmArgs &a, hipStream_t s)
{
    switch (mode) {
    case kFast: return launch_one<BM, BN, WAVES_M, WAVES_N, kFast>(a, s);
    case kVecPred: return launch_one<BM, BN, WAVES_M, WAVES_N, kVecPred>(a, s);
    default: return launch_one<BM, BN, WAVES_M, WAVES_N, kScalar>(a, s);
    }
}

}  // namespace

const char *bf16_kernel_name(int cfg, int mode)
{
    static const char *names[2][3] = {
        {"gemm_bf16_kernel<256, 256, 2, 4, 0>", "gemm_bf16_kernel<256, 256, 2, 4, 1>", "gemm_bf16_kernel<256, 256, 2, 4, 2>"},
        {"gemm_bf16_kernel<128, 128, 2, 2, 0>", "gemm_bf16_kernel<128, 128, 2, 2, 1>", "gemm_bf16_kernel<128, 128, 2, 2, 2>"},
    };
    return cfg == kBf16_Main ? bf16_main_kernel_name() : names[cfg - 1][mode];
}

hipError_t launch_bf16(int cfg, int mode, const GemmArgs &a, hipStream_t s)
{
    switch (cfg) {
    case kBf16_Main: return launch_bf16_main(a, s);
    case kBf16_256x256: return launch_cfg<256, 256, 2, 4>(mode, a, s);
    default: return launch_cfg<128, 128, 2, 2>(mode, a, s);
    }
}

}  // namespace fsrgemm
