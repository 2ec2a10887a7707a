// Main bf16 kernel for large, tile-aligned problems: C[M x N] = A . B with A
// row-major and B column-major (both contiguous along k), fp32 accumulate and
// output -- the Task 2 product at matrix-core input precision.
//
// Shape of the computation
//   workgroup  : 256 lanes = 4 wavefronts, one per SIMD, 256 x 256 tile of C
//   wavefront  : 128 x 128 of that tile = 4 x 4 blocks of V_MFMA_F32_32X32X16_BF16,
//                256 accumulator registers (the whole AccVGPR file)
//   K-tile     : 64 elements = one 128-byte row per tile row, 4 MFMA k-steps
//   LDS        : two stages of (A 32 KB + B 32 KB); stage t%2 is read while
//                stage (t+1)%2 is filled by direct global->LDS loads
//
// A large tile is what keeps the path inside the L2 bandwidth: each K-tile
// moves 64 KB into the workgroup for 33.5 MFLOP.  With one wavefront per SIMD
// nothing else can fill an issue bubble, so the loop is an explicit schedule:
// every MFMA is followed by at most one other instruction (an LDS fragment
// read or a global->LDS load) and the pairs are fenced so the compiler keeps
// that order.  Measured on this part, a 16-byte LDS read in an MFMA's shadow
// costs about 4 cycles and a global->LDS load about 5, while a global load that
// returns into VGPRs stalls the matrix pipe for about 32; hence the operands
// never pass through registers on their way to LDS.
//
// Per K-tile: 64 MFMAs, 32 LDS reads (even slots), 16 global->LDS loads and one
// prefetch touch (odd slots) and one workgroup barrier.  The barrier sits after the third k-step: by then
// this stage's last fragments are in registers and the next stage has landed,
// so the stage just read can be refilled (for K-tile t+2) during the fourth
// k-step and the first k-step of the next K-tile.
//
// That leaves a load roughly three k-steps to arrive, enough for an L2 hit but
// not for a first touch that has to come over the fabric.  Each workgroup
// therefore also touches, several K-tiles ahead, its share of the operand rows
// that the workgroups running beside it on the same XCD read as well (with the
// tile order of tile_coords, 4 neighbours share an A panel and 8 share a B
// panel): one 4-byte global->LDS load per wavefront whose lanes each hit a
// different 128-byte line.  The data is discarded; the lines are then in L2
// when the real loads of all sharers arrive.
//
// LDS rows are 128 bytes, unpadded; 16-byte chunk c of row r is stored at chunk
// position c ^ ((r >> 1) & 7).  A 16-lane group of a 128-bit LDS read then
// touches all 64 banks once (measured: zero bank conflicts).
#include <type_traits>

#include "common.hpp"

namespace fsrgemm {
namespace {

#define FSR_AS1 __attribute__((address_space(1)))
#define FSR_AS3 __attribute__((address_space(3)))

constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kTileBytes = kBM * kBK * 2;       // one operand tile: 32 KB
constexpr int kStageBytes = 2 * kTileBytes;     // A + B: 64 KB
constexpr int kScratchBytes = 1024;             // landing zone of the prefetch touches (256 B per wavefront)
constexpr int kLdsBytes = 2 * kStageBytes + kScratchBytes;
constexpr int kThreads = 256;
constexpr int kEarly = 8;        // loads of a K-tile issued right after the barrier; the other 8 one k-step later
constexpr int kTouchAhead = 3;   // K-tiles between a prefetch touch and the loads it serves: 2 is too late, 4 and
                                 // more let touched lines be evicted before use (more fabric reads, same time)

struct Frag {
    bf16x8 a[4];
    bf16x8 b[4];
};

__global__ __launch_bounds__(kThreads) void gemm_bf16_main_kernel(GemmArgs g, int tiles_m, int tiles_n)
{
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    int tile_m, tile_n;
    tile_coords(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * kBM, n0 = tile_n * kBN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave >> 1) * 128, wn0 = (wave & 1) * 128;
    const int li = lane & 31, lh = lane >> 5;
    const int nk = g.K / kBK;
    const uint16_t *A = static_cast<const uint16_t *>(g.A);
    const uint16_t *B = static_cast<const uint16_t *>(g.B);

    // Global -> LDS.  A load instruction moves 64 x 16 bytes to 1 KB of contiguous LDS = 8 tile rows.
    // Wavefront w fills rows 64 w + 8 q + lane/8 (q = 0..7) of the A tile and of the B tile; the lane
    // fetches the chunk that belongs at its LDS position: (lane % 8) ^ ((row >> 1) & 7).
    const int lrow = lane >> 3, lpos = lane & 7;
    // ((64 w + 8 q + lrow) >> 1) & 7 = 4 (q & 1) + (lrow >> 1): one lane offset for even q, one for odd q
    const int sw_even = (lrow >> 1) & 3, sw_odd = sw_even ^ 4;
    const uint32_t a_lane[2] = {(uint32_t)(lrow * g.lda + (lpos ^ sw_even) * 8) * 2u,
                                (uint32_t)(lrow * g.lda + (lpos ^ sw_odd) * 8) * 2u};
    const uint32_t b_lane[2] = {(uint32_t)(lrow * g.ldb + (lpos ^ sw_even) * 8) * 2u,
                                (uint32_t)(lrow * g.ldb + (lpos ^ sw_odd) * 8) * 2u};
    const char *a_base = reinterpret_cast<const char *>(A + (int64_t)(m0 + wave * 64) * g.lda);
    const char *b_base = reinterpret_cast<const char *>(B + (int64_t)(n0 + wave * 64) * g.ldb);
    const int64_t a_step = 8 * g.lda * 2, b_step = 8 * g.ldb * 2;
    // idx 0..7: A rows 8 idx.., 8..15: B rows 8 (idx-8)...  K-tiles past the end are clamped to the
    // last one: the data lands in a stage that is never read again.
    auto dma = [&](int stage, int idx, int t) {
        const int tc = t < nk ? t : nk - 1;
        const int q = idx & 7;
        char *dst = smem + stage * kStageBytes + (idx < 8 ? 0 : kTileBytes) + (wave * 64 + q * 8) * 128;
        const uint32_t lane_off = idx < 8 ? a_lane[q & 1] : b_lane[q & 1];
        const char *src = (idx < 8 ? a_base + q * a_step : b_base + q * b_step) + (int64_t)tc * (kBK * 2) + lane_off;
        __builtin_amdgcn_global_load_lds((const FSR_AS1 void *)src, (FSR_AS3 void *)dst, 16, 0, 0);
    };

    // Prefetch touches: lanes 0-15 take A rows 64 (tile_n % 4) + 16 w + lane, lanes 16-23 take B rows
    // 32 (tile_m % 8) + 8 w + (lane - 16); the remaining lanes repeat lane 0 and coalesce with it.
    const char *touch_ptr;
    {
        const int tl = lane < 24 ? lane : 0;
        touch_ptr = tl < 16
            ? reinterpret_cast<const char *>(A + (int64_t)(m0 + (tile_n & 3) * 64 + wave * 16 + tl) * g.lda)
            : reinterpret_cast<const char *>(B + (int64_t)(n0 + (tile_m & 7) * 32 + wave * 8 + (tl - 16)) * g.ldb);
    }
    auto touch = [&](int t) {
        const int tc = t < nk ? t : nk - 1;
        __builtin_amdgcn_global_load_lds((const FSR_AS1 void *)(touch_ptr + (int64_t)tc * (kBK * 2)),
                                         (FSR_AS3 void *)(smem + 2 * kStageBytes + wave * 256), 4, 0, 0);
    };

    // Fragment reads: block row li of the wavefront's A (or B) rows, k-chunk 2 kk + lh.
    int ra_off[4], rb_off[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int pos = (2 * kk + lh) ^ ((li >> 1) & 7);
        ra_off[kk] = (wm0 + li) * 128 + pos * 16;
        rb_off[kk] = kTileBytes + (wn0 + li) * 128 + pos * 16;
    }
    Frag F[2];
    // idx orders the eight reads as the next k-step consumes them: a0, b0..b3, a1..a3
    auto lread = [&](int stage, int kk, int fi, int idx) {
        const char *s = smem + stage * kStageBytes;
        if (idx == 0)
            F[fi].a[0] = *reinterpret_cast<const bf16x8 *>(s + ra_off[kk]);
        else if (idx <= 4)
            F[fi].b[idx - 1] = *reinterpret_cast<const bf16x8 *>(s + rb_off[kk] + (idx - 1) * 4096);
        else
            F[fi].a[idx - 4] = *reinterpret_cast<const bf16x8 *>(s + ra_off[kk] + (idx - 4) * 4096);
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // One K-tile t of parity P: reads stage X = P; K-tile t+1 lands in Y = 1-P.  Of K-tile t+1's 16
    // loads the first kEarly were issued in k-step 3 of K-tile t-1, the rest go out in k-step 0 here;
    // k-step 3 starts refilling X with K-tile t+2.
    auto k_tile = [&](auto parity, int t) {
        constexpr int P = decltype(parity)::value;
        constexpr int X = P, Y = 1 - P;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int fc = kk & 1, fn = fc ^ 1;
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                acc[m >> 2][m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(F[fc].a[m >> 2], F[fc].b[m & 3],
                                                                             acc[m >> 2][m & 3], 0, 0, 0);
                if ((m & 1) == 0) {                 // even slots: fragments of the next k-step (next stage after the barrier)
                    if (kk < 3) lread(X, kk + 1, fn, m >> 1); else lread(Y, 0, fn, m >> 1);
                } else {                            // odd slots: loads, so that LDS reads never queue back to back
                    const int c = m >> 1;
                    if (kk == 3) dma(X, c, t + 2);
                    else if (kk == 0) dma(Y, kEarly + c, t + 1);
                    else if (kk == 1 && c == 0) touch(t + kTouchAhead);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (kk == 2) {
                // All loads but the newest (the touch) have landed: K-tile t+1 is complete in Y.  Every
                // wavefront also has its last fragments of X in registers, so after the barrier Y may be
                // read and X overwritten.
                asm volatile("s_waitcnt vmcnt(1) lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // Prologue: K-tile 0 into stage 0 and touches for the K-tiles the loop's own touches come too late for;
    // only K-tile 0 is waited for (the touches are the youngest kTouchAhead - 1 loads).
#pragma unroll
    for (int idx = 0; idx < 16; ++idx) dma(0, idx, 0);
#pragma unroll
    for (int p = 1; p < kTouchAhead; ++p) touch(p);
    static_assert(kTouchAhead == 3, "the wait below skips kTouchAhead - 1 touches");
    asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // then the early half of K-tile 1 into stage 1 and the first fragments
#pragma unroll
    for (int idx = 0; idx < kEarly; ++idx) dma(1, idx, 1);
#pragma unroll
    for (int idx = 0; idx < 8; ++idx) lread(0, 0, 0, idx);
    __builtin_amdgcn_sched_barrier(0);

    int t = 0;
    for (; t + 1 < nk; t += 2) {
        k_tile(std::integral_constant<int, 0>{}, t);
        k_tile(std::integral_constant<int, 1>{}, t + 1);
    }
    if (t < nk) k_tile(std::integral_constant<int, 0>{}, t);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // no load may still be writing LDS when the wavefront ends

    // Register r of a 32x32 block holds row (r/4)*8 + 4*(lane/32) + r%4, column lane%32.
    float *__restrict__ C = g.C;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = n0 + wn0 + j * 32 + li;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm0 + i * 32 + (r / 4) * 8 + lh * 4 + (r % 4);
                C[(int64_t)row * g.ldc + col] = acc[i][j][r];
            }
        }
}

}  // namespace

const char *bf16_main_kernel_name() { return "gemm_bf16_main_kernel"; }

// Requires M % 256 == 0, N % 256 == 0, K % 64 == 0, K >= 64, 16-byte aligned bases,
// lda % 8 == 0, ldb % 8 == 0 and leading dimensions below 2^25 (32-bit lane offsets).
hipError_t launch_bf16_main(const GemmArgs &a, hipStream_t s)
{
    static std::atomic<uint64_t> configured{0};
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(gemm_bf16_main_kernel), kLdsBytes, configured);
    if (e != hipSuccess) return e;
    const int tiles_m = a.M / kBM, tiles_n = a.N / kBN;
    hipLaunchKernelGGL(gemm_bf16_main_kernel, dim3((unsigned)(tiles_m * tiles_n)), dim3(kThreads), kLdsBytes, s, a,
                       tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace fsrgemm
