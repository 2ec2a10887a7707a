// bf16 x bf16 -> fp32 GEMM for gfx950: C[M x N] = A[M x K] . B[K x N], C row-major
// fp32, each operand in either storage order (the same product as the paper's
// Task 2, at the reduced input precision that matrix cores are built for;
// accumulation and output stay fp32).
//
// This file holds the general-purpose kernel: any shape, any alignment, any
// storage order, three tile sizes.  Large aligned problems go to the kernel in
// gemm_bf16_main.hip.
//
// One workgroup of 256 lanes (4 wavefronts, 2 x 2) owns a (64 T) x (64 T) tile
// of C, each wavefront 2T x 2T blocks of V_MFMA_F32_16X16X32_BF16: lane l
// supplies eight consecutive k (16 bytes) of row l % 16, k-offset 8 * (l / 16),
// for each operand -- one 16-byte LDS read per operand block and k-step of 32.
// Per K-tile of 64 (one 128-byte row per tile row, two k-steps) A[BM x 64] and
// B^T[BN x 64] are staged through registers into double-buffered LDS; staging
// through registers is what lets ragged edges be zero-filled lane by lane and
// lets an operand that is contiguous along m / n be transposed on the way: a
// lane then loads an 8-row x NV-k block as NV vectors of 8 rows, regroups the
// 16-bit values in registers and stores 8 row pieces of NV k.
//
// LDS rows are 128 bytes with no padding; the 16-byte chunk c of row r is kept
// at chunk position c ^ ((r >> 1) & 7), so that the 16 rows that one group of
// lanes reads at one k-offset cover all 64 banks exactly once.
//
// The loop is an explicit schedule, fenced so the compiler keeps it: the MFMAs
// of a k-step carry, evenly spread, the fragment reads of the next k-step and
// either the LDS stores of the next K-tile (k-step 0) or the global loads of the
// one after (k-step 1, each register reloaded only after it has been stored).
// The one barrier per K-tile sits between the k-steps: the last fragments of
// this stage are in registers by then and the next stage is completely written.
// Of the three load modes (as in gemm_f32.hip), the two checked ones let a
// workgroup whose tile lies inside the matrix load its whole K-tiles unchecked
// (from merely element-aligned addresses in the unaligned mode); only the
// ragged end of K and matrices narrower than a tile pay for checks.
// The MFMAs are inline assembly so that every accumulator block stays in its
// registers across the loop (see gemm_bf16_main.hip); a block is touched again
// NB * NB >= 4 MFMAs later and the epilogue starts behind explicit wait states.
#include <stdio.h>

#include <type_traits>

#include "launchers.hpp"

namespace fsrgemm {
namespace {

constexpr int kThreads = 256;
constexpr int kBK = 64;                 // bf16 elements per K-tile: one 128-byte row
constexpr int kRowBytes = kBK * 2;

template <int MODE>
__device__ __forceinline__ u32x4 load8(const uint16_t *__restrict__ p, bool row_ok, int col, int col_limit)
{
    // p points at element (row, col) of the stored matrix; the vector covers col .. col+7 of that row.
    if constexpr (MODE == kFast) {
        return *reinterpret_cast<const u32x4 *>(p);
    } else if constexpr (MODE == kUnalignedVec) {
        u32x4 v;
        __builtin_memcpy(&v, p, sizeof v);
        return v;
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

// A lane's share of one operand tile (EXT rows of m or n, 64 k) on its way global -> registers -> LDS.
// NV = EXT / 32 vectors of 16 bytes per lane either way.
//   kKContig : vector s = row (tid >> 3) + 32 s of the tile, 16-byte chunk tid & 7 of its 64 k: stored as loaded
//   kMnContig: the lane owns rows 8 rb .. 8 rb + 7 and k = NV kg .. NV kg + NV - 1 (kg = tid % (64 / NV),
//              rb = tid / (64 / NV)); vector s holds those 8 rows at k = NV kg + s.  Eight row pieces of NV k
//              (2 NV bytes) go to LDS, `8 / NV` of them per store step so that both layouts take NV steps.
template <int EXT, int LAY>
struct Staging {
    static constexpr int NV = EXT / 32;
    static constexpr int KG = kBK / NV;

    template <int MODE>
    static __device__ __forceinline__ u32x4 gload(const uint16_t *__restrict__ base, int64_t ld, int r0, int rows, int k0,
                                                  int K, int tid, int s)
    {
        if constexpr (LAY == kKContig) {
            const int r = (tid >> 3) + 32 * s, k = (tid & 7) * 8;
            return load8<MODE>(base + (int64_t)(r0 + r) * ld + k0 + k, r0 + r < rows, k0 + k, K);
        } else {
            const int r = 8 * (tid / KG), k = NV * (tid % KG) + s;
            return load8<MODE>(base + (int64_t)(k0 + k) * ld + r0 + r, k0 + k < K, r0 + r, rows);
        }
    }
    // store step s of this operand; v = the lane's NV vectors, tile = LDS address of the operand tile's stage
    static __device__ __forceinline__ void lstore(char *tile, const u32x4 *v, int tid, int s)
    {
        if constexpr (LAY == kKContig) {
            const int r = (tid >> 3) + 32 * s, c = tid & 7;
            *reinterpret_cast<u32x4 *>(tile + r * kRowBytes + ((c ^ ((r >> 1) & 7)) * 16)) = v[s];
        } else {
            const int kb = NV * (tid % KG) * 2;         // byte offset of the lane's k range inside a row
#pragma unroll
            for (int i = s * (8 / NV); i < (s + 1) * (8 / NV); ++i) {
                const int r = 8 * (tid / KG) + i;
                uint32_t w[NV / 2];
#pragma unroll
                for (int j = 0; j < NV / 2; ++j) {      // k = 2j, 2j + 1 of row i: one half of a dword from each vector
                    const uint32_t x = v[2 * j][i >> 1], y = v[2 * j + 1][i >> 1];
                    w[j] = (i & 1) ? (x >> 16) | (y & 0xFFFF0000u) : (x & 0xFFFFu) | (y << 16);
                }
                char *p = tile + r * kRowBytes + (((kb >> 4) ^ ((r >> 1) & 7)) * 16) + (kb & 15);
                if constexpr (NV == 8) *reinterpret_cast<u32x4 *>(p) = u32x4{w[0], w[1], w[2], w[3]};
                else if constexpr (NV == 4) *reinterpret_cast<uint2 *>(p) = uint2{w[0], w[1]};
                else *reinterpret_cast<uint32_t *>(p) = w[0];
            }
        }
    }
};

template <int T, int MIN_WAVES, int MODE, int ALAY, int BLAY>
__global__ __launch_bounds__(kThreads, MIN_WAVES) void gemm_bf16_kernel(GemmArgs g, int tiles_m, int tiles_n)
{
    constexpr int BM = 64 * T, BN = 64 * T;
    constexpr int TILE_B = BM * kRowBytes;          // bytes of one operand tile
    constexpr int STAGE_B = 2 * TILE_B;             // A + B
    constexpr int NV = BM / 32;                     // 16-byte vectors per lane per operand and K-tile
    constexpr int NG = 2 * NV;                      // ... of both operands
    constexpr int NB = 2 * T;                       // 16-row blocks per wavefront and operand
    constexpr int NR = 2 * NB;                      // fragment reads per k-step; equals NG
    constexpr int NMF = NB * NB;                    // MFMAs per k-step
    constexpr int NC = NR + NG;                     // companion instructions per k-step, alternating read / memory
    static_assert(NR == NG, "reads and memory operations alternate");
    using StA = Staging<BM, ALAY>;
    using StB = Staging<BN, BLAY>;

    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const uint16_t *__restrict__ A = static_cast<const uint16_t *>(g.A);
    const uint16_t *__restrict__ B = static_cast<const uint16_t *>(g.B);
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
    const int wm0 = (wave >> 1) * 32 * T, wn0 = (wave & 1) * 32 * T;
    const int l16 = lane & 15, lq = lane >> 4;

    if (nk == 0) {      // K == 0 (or a slice past the end of K): every entry is an empty sum
        for (int e = tid; e < BM * BN; e += kThreads) {
            const int row = m0 + e / BN, col = n0 + e % BN;
            if (row < M && col < N) C[(int64_t)row * g.ldc + col] = 0.f;
        }
        return;
    }

    // A workgroup whose tile lies inside the matrix needs no check on whole K-tiles even when the problem as a
    // whole is ragged: `unchecked` counts the leading K-tiles it may load like the unchecked mode does.
    const int unchecked = MODE == kFast ? nk : (m0 + BM <= M && n0 + BN <= N) ? max(0, min(nk, K / kBK - t0)) : 0;
    u32x4 rg[NG];       // idx < NV: A's vectors; else B's
    auto gload = [&](auto load_mode, int idx, int t) {      // K-tiles past the end are clamped: loaded again, never consumed
        constexpr int LM = decltype(load_mode)::value;
        const int k0 = (t0 + (t < nk ? t : nk - 1)) * kBK;
        if (idx < NV) rg[idx] = StA::template gload<LM>(A, g.lda, m0, M, k0, K, tid, idx);
        else rg[idx] = StB::template gload<LM>(B, g.ldb, n0, N, k0, K, tid, idx - NV);
    };
    using Checked = std::integral_constant<int, MODE>;
    using Unchecked = std::integral_constant<int, MODE == kScalar ? kUnalignedVec : kFast>;
    auto lwrite = [&](int stage, int idx) {
        if (idx < NV) StA::lstore(smem + stage * STAGE_B, rg, tid, idx);
        else StB::lstore(smem + stage * STAGE_B + TILE_B, rg + NV, tid, idx - NV);
    };
    // Fragment of 16 rows x 32 k: the lane reads row l16 of the block, 16-byte chunk 4 kk + lq.
    const int ra0 = (wm0 + l16) * kRowBytes, rb0 = TILE_B + (wn0 + l16) * kRowBytes;
    const int rsw = (l16 >> 1) & 7;
    bf16x8 fa[2][NB], fb[2][NB];
    auto lread = [&](int stage, int kk, int idx) {    // into the fragments of k-step kk; idx < NB: A block idx; else B block
        const int pos = ((4 * kk + lq) ^ rsw) * 16;
        const char *s = smem + stage * STAGE_B + pos;
        if (idx < NB) fa[kk][idx] = *reinterpret_cast<const bf16x8 *>(s + ra0 + idx * 16 * kRowBytes);
        else fb[kk][idx - NB] = *reinterpret_cast<const bf16x8 *>(s + rb0 + (idx - NB) * 16 * kRowBytes);
    };

    f32x4 acc[NB][NB];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // K-tile t of parity P reads stage X = P; K-tile t+1 (in rg) is stored to Y = 1-P during k-step 0,
    // rg is refilled with K-tile t+2 during k-step 1.
    auto k_tile = [&](auto parity, auto load_mode, int t) {
        constexpr int P = decltype(parity)::value;
        constexpr int X = P, Y = 1 - P;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
            for (int m = 0; m < NMF; ++m) {
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0"
                             : "+a"(acc[m / NB][m % NB])
                             : "v"(fa[kk][m / NB]), "v"(fb[kk][m % NB]));
#pragma unroll
                for (int c = m * NC / NMF; c < (m + 1) * NC / NMF; ++c) {
                    const int q = c >> 1;
                    if ((c & 1) == 0) {
                        if (kk == 0) lread(X, 1, q); else lread(Y, 0, q);
                    } else {
                        if (kk == 0) lwrite(Y, q); else gload(load_mode, q, t + 2);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (kk == 0) {
                __builtin_amdgcn_s_waitcnt(0xC07F);         // lgkmcnt(0): this wavefront's LDS stores and reads are done
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // Prologue: K-tile 0 through the registers into stage 0, K-tile 1 into the registers, first fragments.
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
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int idx = 0; idx < NR; ++idx) lread(0, 0, idx);
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
    // the last MFMAs must have retired before the accumulators are read (the compiler does not know what wrote them)
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");

    // Register r of a 16x16 block holds row 4 (lane / 16) + r, column lane % 16.
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int col = n0 + wn0 + j * 16 + l16;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = m0 + wm0 + i * 16 + lq * 4 + r;
                if (MODE == kFast || (row < M && col < N)) C[(int64_t)row * g.ldc + col] = acc[i][j][r];
            }
        }
}

template <int T, int MIN_WAVES, int MODE, int ALAY, int BLAY>
hipError_t launch_one(const GemmArgs &a, hipStream_t s)
{
    constexpr int BM = 64 * T;
    constexpr int lds = 2 * 2 * BM * kRowBytes;
    auto kern = gemm_bf16_kernel<T, MIN_WAVES, MODE, ALAY, BLAY>;
    static std::atomic<uint64_t> configured{0};
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds, configured);
    if (e != hipSuccess) return e;
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BM - 1) / BM;
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n * a.k_slices)), dim3(kThreads), lds, s, a, tiles_m, tiles_n);
    return hipGetLastError();
}

template <int T, int MIN_WAVES, int ALAY, int BLAY>
hipError_t launch_lay(int mode, const GemmArgs &a, hipStream_t s)
{
    switch (mode) {
    case kFast: return launch_one<T, MIN_WAVES, kFast, ALAY, BLAY>(a, s);
    case kVecPred: return launch_one<T, MIN_WAVES, kVecPred, ALAY, BLAY>(a, s);
    default: return launch_one<T, MIN_WAVES, kScalar, ALAY, BLAY>(a, s);
    }
}

template <int T, int MIN_WAVES>
hipError_t launch_cfg(int mode, int a_lay, int b_lay, const GemmArgs &a, hipStream_t s)
{
    if (a_lay == kKContig) {
        return b_lay == kKContig ? launch_lay<T, MIN_WAVES, kKContig, kKContig>(mode, a, s)
                                 : launch_lay<T, MIN_WAVES, kKContig, kMnContig>(mode, a, s);
    }
    return b_lay == kKContig ? launch_lay<T, MIN_WAVES, kMnContig, kKContig>(mode, a, s)
                             : launch_lay<T, MIN_WAVES, kMnContig, kMnContig>(mode, a, s);
}

}  // namespace

// <T, minimum wavefronts per SIMD, load mode, A layout, B layout>: tile (64 T) x (64 T); as a profiler trace prints it
const char *bf16_kernel_name(int cfg, int mode, int a_lay, int b_lay)
{
    struct Names {
        char text[3][3][2][2][40];
        Names()
        {
            static const char *shapes[3] = {"4, 1", "2, 2", "1, 4"};
            for (int c = 0; c < 3; ++c)
                for (int m = 0; m < 3; ++m)
                    for (int x = 0; x < 2; ++x)
                        for (int y = 0; y < 2; ++y)
                            snprintf(text[c][m][x][y], sizeof text[c][m][x][y], "gemm_bf16_kernel<%s, %d, %d, %d>", shapes[c],
                                     m, x, y);
        }
    };
    static const Names names;
    return bf16_main_shape(cfg) >= 0 ? bf16_main_kernel_name(bf16_main_shape(cfg), a_lay, b_lay) : names.text[cfg - 1][mode][a_lay][b_lay];
}

hipError_t launch_bf16(int cfg, int mode, int a_lay, int b_lay, const GemmArgs &a, hipStream_t s)
{
    if (bf16_main_shape(cfg) >= 0) return launch_bf16_main(bf16_main_shape(cfg), a_lay, b_lay, a, s);
    switch (cfg) {
    case kBf16_256x256: return launch_cfg<4, 1>(mode, a_lay, b_lay, a, s);
    case kBf16_128x128: return launch_cfg<2, 2>(mode, a_lay, b_lay, a, s);
    default: return launch_cfg<1, 4>(mode, a_lay, b_lay, a, s);
    }
}

}  // namespace fsrgemm
