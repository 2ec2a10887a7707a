// fp32 kernel for large, aligned problems: C[M x N] = A . B with fp32 operands, accumulation and output (the
// paper's Task 2 at its own precision), one 256 x 256 tile of C per workgroup and direct global->LDS loads.
// Either operand may be contiguous along k (a row-major A, a B stored transposed: a tile row is 128 bytes of
// 32 k) or along m / n (an A stored transposed, a row-major B: a tile row is a k-row of 1 KB); LDS keeps the
// memory order and the fragment reads do the rest.
//
// Shape of the computation
//   workgroup : 256 lanes = 4 wavefronts, one per SIMD
//   wavefront : 128 x 128 of the tile = 4 x 4 blocks of V_MFMA_F32_32X32X2_F32, 256 accumulator registers (the
//               whole AccVGPR file)
//   K-tile    : 32 elements = 16 MFMA k-steps of 2, taken as 4 chunks of 8 k (64 MFMAs each)
//   LDS       : two stages of (A 32 KB + B 32 KB)
//
// Against the 256 x 128 tiles of the general kernel a K-tile here feeds twice the flops per byte brought into
// the compute unit (64 flops per byte), and with a 64-cycle MFMA one wavefront per SIMD keeps the matrix core
// busy on its own: everything else -- 8 to 32 LDS fragment reads per chunk, 16 global->LDS loads per K-tile --
// is issued in the shadow of the MFMAs, one instruction behind each, in an order fixed with scheduling fences.
//
// Pipeline, per K-tile t held in stage t % 2:
//   chunks 0..2 : MFMAs of the chunk; the fragments of the next chunk are read from the same stage
//   end of chunk 2 : every fragment of this stage is in registers and K-tile t + 1 has landed in the other stage
//               (waits on this wavefront's reads and loads, then the one barrier of the K-tile)
//   chunk 3     : MFMAs; the first fragments of K-tile t + 1 are read from the other stage, and the loads of
//               K-tile t + 2 are issued into this one, which nobody reads any more.  Two loads never sit behind
//               consecutive MFMAs: a load that finds the address path busy holds up the wavefront, MFMAs included.
// So no MFMA ever waits for LDS latency behind the barrier, and a load has three quarters of a K-tile (about
// 5 us) to land.
//
// The loads are issued by hand in their scalar-base form: a wavefront-uniform 64-bit base in scalar registers
// (computed by the scalar unit beside the MFMAs) plus one 32-bit lane offset register that never changes.  Issued
// through the compiler's builtin with a 64-bit address per lane, each load held the matrix pipe up for about 24
// cycles (147 TFLOP/s on 4096^3 instead of 150).
//
// The MFMAs are inline assembly with "+a" operands so that every accumulator block stays in its registers across
// the loop's back edge; the compiler does not know they are MFMAs, so the wait before the accumulators are
// read at the end is written out.
//
// LDS layout of an operand's 32 KB:
//   contiguous along k   : 256 rows of 128 bytes; the 16-byte piece c of row r sits at position
//                          c ^ ((r >> 1) & 7), which makes the 16-byte fragment reads (32 rows x 2 pieces per
//                          wavefront) conflict-free
//   contiguous along m/n : 32 k-rows of 1 KB; piece c of k-row k sits at position c ^ (8 * (k & 1))
// A global->LDS load writes its 64 lanes' 16 bytes to consecutive LDS addresses, so the permutation is applied
// on the global side: the lane that fills position p fetches the piece that belongs there.
#include <type_traits>

#include "launchers.hpp"

namespace fsrgemm {

namespace {

constexpr int kBM = 256, kBN = 256, kBK = 32, kThreads = 256;
constexpr int kOperandBytes = 256 * kBK * 4;                // 32 KB, either layout
constexpr int kStageBytes = 2 * kOperandBytes;
constexpr int kLdsBytes = 2 * kStageBytes;                  // 128 KB

#define FENCE() __builtin_amdgcn_sched_barrier(0)
#define GLOBAL_PTR __attribute__((address_space(1)))
#define LDS_PTR __attribute__((address_space(3)))

template <int ALAY, int BLAY>
__global__ __launch_bounds__(kThreads, 1) void gemm_f32_main_kernel(GemmArgs g, int tiles_m, int tiles_n)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    int tile_m, tile_n;
    tile_coords(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_origin(tile_m, kBM, g.M), n0 = tile_origin(tile_n, kBN, g.N);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm0 = (wave >> 1) * 128, wn0 = (wave & 1) * 128;
    const int li = lane & 31, lh = lane >> 5;
    const int nk = g.K / kBK;
    const float *__restrict__ A = static_cast<const float *>(g.A);
    const float *__restrict__ B = static_cast<const float *>(g.B);

    // Load q (0..7) of wavefront w for an operand fills the LDS bytes [(8 w + q) KB, +1 KB) of the operand:
    //   along k   : rows 64 w + 8 q + lane / 8, position lane % 8, which holds piece
    //               (lane % 8) ^ ((row >> 1) & 7) with (row >> 1) & 7 = 4 (q & 1) + (lane >> 4)
    //   along m/n : k-row 8 w + q, position lane, which holds piece lane ^ (8 * (q & 1))
    // K-tiles beyond the last one (the pipeline asks for two ahead) repeat the last: in bounds and never read.
    // The address of a load is a wavefront-uniform pointer (scalar arithmetic, free beside the MFMAs) plus a 32-bit
    // lane offset that is fixed for the whole kernel: two per operand, by the parity of q.
    auto lane_offset = [&](auto layout, int64_t ld, int odd) -> uint32_t {
        constexpr int LAY = decltype(layout)::value;
        if constexpr (LAY == kKContig) return (uint32_t)(((lane >> 3) * ld + (((lane & 7) ^ ((4 * odd + (lane >> 4)) & 7)) << 2)) << 2);
        else return (uint32_t)((lane ^ (8 * odd)) << 4);
    };
    const uint32_t a_off[2] = {lane_offset(std::integral_constant<int, ALAY>{}, g.lda, 0), lane_offset(std::integral_constant<int, ALAY>{}, g.lda, 1)};
    const uint32_t b_off[2] = {lane_offset(std::integral_constant<int, BLAY>{}, g.ldb, 0), lane_offset(std::integral_constant<int, BLAY>{}, g.ldb, 1)};
    // A load is issued by hand in two steps: M0 <- its LDS address, then, at least one instruction later (M0 needs a
    // wait state before a load reads it), the load in its scalar-base form.
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(LDS_PTR char *)lds);
    auto load_m0 = [&](int stage, int idx) {       // idx 0..15: A and B loads alternate, q = idx / 2
        const uint32_t dst = lds0 + stage * kStageBytes + (idx & 1) * kOperandBytes + (wave * 8 + (idx >> 1)) * 1024;
        asm volatile("s_mov_b32 m0, %0" ::"s"(dst) : "m0");
    };
    auto dma = [&](auto layout, const float *__restrict__ P, int64_t ld, int origin, const uint32_t (&off)[2], int q, int t) {
        constexpr int LAY = decltype(layout)::value;
        const int tc = t < nk ? t : nk - 1;
        const float *row;       // uniform
        if constexpr (LAY == kKContig) row = P + (int64_t)(origin + wave * 64 + 8 * q) * ld + tc * kBK;
        else row = P + (int64_t)(tc * kBK + wave * 8 + q) * ld + origin;
        asm volatile("global_load_lds_dwordx4 %0, %1" ::"v"(off[q & 1]), "s"(row) : "memory");
    };
    auto load_go = [&](int idx, int t) {
        if (idx & 1) dma(std::integral_constant<int, BLAY>{}, B, g.ldb, n0, b_off, idx >> 1, t);
        else dma(std::integral_constant<int, ALAY>{}, A, g.lda, m0, a_off, idx >> 1, t);
    };
    auto load = [&](int stage, int idx, int t) {    // outside the MFMA loop
        load_m0(stage, idx);
        asm volatile("s_nop 0" ::: "memory");
        load_go(idx, t);
    };

    // Fragments of chunk c (8 k): the lane with row / column x = offset + 32 block + lane % 32 holds
    // k = 8 c + 4 (lane / 32) + s for the four steps s of the chunk -- one 16-byte read along k, four 4-byte
    // reads along m / n.
    float fa[2][4][4], fb[2][4][4];         // [register buffer][block][step]
    constexpr int kReadsA = ALAY == kKContig ? 4 : 16, kReadsB = BLAY == kKContig ? 4 : 16;
    auto fragment = [&](auto layout, int operand, int offset, int stage, int c, float (&f)[4][4], int idx) {
        constexpr int LAY = decltype(layout)::value;
        const char *st = lds + stage * kStageBytes + operand * kOperandBytes;
        if constexpr (LAY == kKContig) {
            const int b = idx;
            const f32x4 v = *reinterpret_cast<const f32x4 *>(st + (offset + 32 * b + li) * 128 + (((2 * c + lh) ^ ((li >> 1) & 7)) << 4));
#pragma unroll
            for (int s = 0; s < 4; ++s) f[b][s] = v[s];
        } else {
            const int b = idx & 3, s = idx >> 2;
            const int k = 8 * c + 4 * lh + s, x = offset + 32 * b + li;
            f[b][s] = *reinterpret_cast<const float *>(st + k * 1024 + ((((x >> 2) ^ (8 * (k & 1))) << 4) | ((x & 3) << 2)));
        }
    };
    auto read = [&](int stage, int c, int buf, int idx) {   // idx 0 .. kReadsA + kReadsB - 1
        if (idx < kReadsA) fragment(std::integral_constant<int, ALAY>{}, 0, wm0, stage, c, fa[buf], idx);
        else fragment(std::integral_constant<int, BLAY>{}, 1, wn0, stage, c, fb[buf], idx - kReadsA);
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
            asm volatile("" : "+a"(acc[i][j]));
        }

    // K-tiles 0 and 1 into stages 0 and 1, then the first fragments
#pragma unroll
    for (int idx = 0; idx < 16; ++idx) load(0, idx, 0);
#pragma unroll
    for (int idx = 0; idx < 16; ++idx) load(1, idx, 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    FENCE();
#pragma unroll
    for (int idx = 0; idx < kReadsA + kReadsB; ++idx) read(0, 0, 0, idx);
    FENCE();

    auto k_tile = [&](auto parity, int t) {
        constexpr int X = decltype(parity)::value, Y = 1 - X;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int cur = c & 1, nxt = cur ^ 1;
#pragma unroll
            for (int m = 0; m < 64; ++m) {
                const int s = m >> 4, i = (m >> 2) & 3, j = m & 3;
                const bool loads = c == 3 && m >= 32 && !(m & 1);
                if (loads) load_m0(X, (m - 32) >> 1);
                {
                    const float av = fa[cur][i][s], bv = fb[cur][j][s];
                    asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(av), "v"(bv));
                }
                if (loads) load_go((m - 32) >> 1, t + 2);
                if (m < kReadsA + kReadsB) {
                    if (c < 3) read(X, c + 1, nxt, m);
                    else read(Y, 0, nxt, m);
                }
                FENCE();
            }
            if (c == 2) {
                asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                FENCE();
            }
        }
    };
    int t = 0;
    for (; t + 1 < nk; t += 2) {
        k_tile(std::integral_constant<int, 0>{}, t);
        k_tile(std::integral_constant<int, 1>{}, t + 1);
    }
    if (t < nk) k_tile(std::integral_constant<int, 0>{}, t);

    // Every global->LDS load has landed before the workgroup gives up its LDS, and the last MFMAs (64 cycles each,
    // unknown to the compiler as such) have written their accumulators before these are read.
    asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = n0 + wn0 + j * 32 + li;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm0 + i * 32 + (r / 4) * 8 + lh * 4 + (r % 4);
                g.C[(int64_t)row * g.ldc + col] = acc[i][j][r];
            }
            FENCE();
        }
}

template <int ALAY, int BLAY>
hipError_t launch_main(const GemmArgs &a, hipStream_t s)
{
    auto kern = gemm_f32_main_kernel<ALAY, BLAY>;
    static std::atomic<uint64_t> configured{0};
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), kLdsBytes, configured);
    if (e != hipSuccess) return e;
    const int tiles_m = (a.M + kBM - 1) / kBM, tiles_n = (a.N + kBN - 1) / kBN;
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(kThreads), kLdsBytes, s, a, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

// <A layout, B layout> with 0 = contiguous along k, 1 = along m / n; as a profiler trace prints the kernel
const char *f32_main_kernel_name(int a_lay, int b_lay)
{
    static const char *names[2][2] = {{"gemm_f32_main_kernel<0, 0>", "gemm_f32_main_kernel<0, 1>"},
                                      {"gemm_f32_main_kernel<1, 0>", "gemm_f32_main_kernel<1, 1>"}};
    return names[a_lay][b_lay];
}

// Whole unchecked 256 x 256 x 32 tiles of 16-byte pieces: a matrix at least one tile high and wide (a ragged
// last tile is shifted back into it), whole K-tiles, 16-byte aligned bases and rows, and, for an operand that is
// contiguous along m (n), M (N) a multiple of 4 so that a shifted tile still starts on a piece.
bool f32_main_fits(int a_lay, int b_lay, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb)
{
    const bool aligned = ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 15u) == 0 && lda % 4 == 0 && ldb % 4 == 0;
    return aligned && M >= kBM && N >= kBN && K >= kBK && K % kBK == 0 && (a_lay == kKContig || M % 4 == 0) &&
           (b_lay == kKContig || N % 4 == 0) && ((M + kBM - 1) / kBM) * ((N + kBN - 1) / kBN) < ((int64_t)1 << 31);
}

// requires f32_main_fits(...) and a.k_slices == 1
hipError_t launch_f32_main(int a_lay, int b_lay, const GemmArgs &a, hipStream_t s)
{
    if (!f32_main_fits(a_lay, b_lay, a.M, a.N, a.K, a.A, a.lda, a.B, a.ldb) || a.k_slices != 1) return hipErrorInvalidValue;
    if (a_lay == kKContig) return b_lay == kKContig ? launch_main<kKContig, kKContig>(a, s) : launch_main<kKContig, kMnContig>(a, s);
    return b_lay == kKContig ? launch_main<kMnContig, kKContig>(a, s) : launch_main<kMnContig, kMnContig>(a, s);
}

}  // namespace fsrgemm
