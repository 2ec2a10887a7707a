// fp32 kernel for large, aligned problems: C[M x N] = A . B with fp32 operands, accumulation and output (the
// paper's Task 2 at its own precision), one 256 x 256 tile of C per workgroup -- or a smaller one, see "Tile
// shapes" -- and direct global->LDS loads.
// Either operand may be contiguous along k (a row-major A, a B stored transposed: a tile row is 128 bytes of
// 32 k) or along m / n (an A stored transposed, a row-major B: a tile row is a k-row of 1 KB); LDS keeps the
// memory order and the fragment reads do the rest.
//
// Shape of the computation (for the 256 x 256 tile)
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
// LDS layout of an operand's tile (32 KB for 256 rows or columns):
//   contiguous along k   : rows of 128 bytes; the 16-byte piece c of row r sits at position c ^ ((r >> 1) & 7),
//                          which makes the 16-byte fragment reads (32 rows x 2 pieces per wavefront) conflict-free
//   contiguous along m/n : 32 k-rows as in memory (1 KB for 256 columns); the 4-byte fragment reads take 32
//                          consecutive words per half wavefront and need no permutation
// A global->LDS load writes its 64 lanes' 16 bytes to consecutive LDS addresses, so the permutation is applied
// on the global side: the lane that fills position p fetches the piece that belongs there.
//
// Tile shapes.  A launch lasts as long as the compute unit with the most tiles, so a problem whose 256 x 256 tiles
// do not fill whole rounds of the 256 compute units is better off with a smaller tile that does: the kernel is a
// template over the blocks per wavefront, WM x WN of 32 x 32 (tile 64 WM x 64 WN), instantiated for the nine shapes
// with sides of 256, 192 and 128 and for 64 x 64, 128 x 64 and 64 x 128, which small problems need to give every
// compute unit a tile (several of these small workgroups share a compute unit: 32 to 48 KB of LDS and under 100
// registers each).  Loads per wavefront and K-tile: 2 WM + 2 WN.
#include <stdio.h>

#include <type_traits>

#include "launchers.hpp"

namespace fsrgemm {

namespace {

constexpr int kBK = 32, kThreads = 256;

// k per slice when K is cut into `slices`: a whole number of K-tiles, the last slice takes what is left
__host__ __device__ constexpr int main_slice_length(int K, int slices) { return ((K + kBK - 1) / kBK + slices - 1) / slices * kBK; }

#define FENCE() __builtin_amdgcn_sched_barrier(0)
#define LDS_PTR __attribute__((address_space(3)))
#define GLOBAL_PTR __attribute__((address_space(1)))

// where the loads of the last, partial K-tile fetch the pieces that lie beyond K
__device__ __attribute__((aligned(16))) const float kZeroPiece[4] = {0.f, 0.f, 0.f, 0.f};

// M0 is on a clobber list below on purpose (the loads take their LDS address from it); clang warns that it is a
// reserved register.  Nothing the compiler emits for this kernel uses M0.
#pragma clang diagnostic ignored "-Winline-asm"

template <int WM, int WN, int ALAY, int BLAY>
__global__ __launch_bounds__(kThreads, 1) void gemm_f32_main_kernel(GemmArgs g, int tiles_m, int tiles_n)
{
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int kBytesA = BM * kBK * 4, kBytesB = BN * kBK * 4, kStageBytes = kBytesA + kBytesB;
    constexpr int kLoadsA = 2 * WM, kLoadsB = 2 * WN, kLoads = kLoadsA + kLoadsB;     // 1 KB each, per wavefront and K-tile
    constexpr int kMfmas = 4 * WM * WN;                                               // per chunk of 8 k
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    // K slices (a call with a workspace): workgroup ids beyond the first tiles_m * tiles_n belong to further slices.
    // Slice s is the product over k in [s per, s per + its length) with per a whole number of K-tiles, written to the
    // s-th M x N block behind g.C (the workspace, tightly packed: the launcher sets ldc = N): for the rest of the kernel
    // it is simply a product of its own, on operands shifted along k.
    int pid = blockIdx.x;
    if (g.k_slices > 1) {
        const int tiles = tiles_m * tiles_n, slice = pid / tiles;
        pid -= slice * tiles;
        const int per = main_slice_length(g.K, g.k_slices), k0 = slice * per;
        g.A = static_cast<const float *>(g.A) + (ALAY == kKContig ? (int64_t)k0 : (int64_t)k0 * g.lda);
        g.B = static_cast<const float *>(g.B) + (BLAY == kKContig ? (int64_t)k0 : (int64_t)k0 * g.ldb);
        g.K = min(per, g.K - k0);
        g.C += (int64_t)slice * g.slice_stride;
    }
    int tile_m, tile_n;
    tile_coords(pid, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_origin(tile_m, BM, g.M), n0 = tile_origin(tile_n, BN, g.N);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm0 = (wave >> 1) * 32 * WM, wn0 = (wave & 1) * 32 * WN;
    const int li = lane & 31, lh = lane >> 5;
    const int nk = g.K / kBK;
    const float *__restrict__ A = static_cast<const float *>(g.A);
    const float *__restrict__ B = static_cast<const float *>(g.B);

    // Load q of wavefront w for an operand of EXT rows / columns (q < EXT / 32) fills the LDS bytes
    // [(w EXT / 32 + q) KB, +1 KB) of the operand's tile:
    //   along k   : rows w EXT / 4 + 8 q + lane / 8, position lane % 8, which holds piece
    //               (lane % 8) ^ ((row >> 1) & 7) with (row >> 1) & 7 = (4 q + (lane >> 4)) & 7
    //   along m/n : k-rows of 4 EXT bytes, stored back to back.  The load starts (1024 q) mod (4 EXT) bytes into k-row
    //               (w EXT / 32 + q) 256 / EXT (rounded down) and runs on into the next k-row where that one ends:
    //               1 KB is one k-row of 256 columns, two of 128, and one and a third of 192, where the start
    //               takes three values in turn
    // The address of a load is a wavefront-uniform pointer (scalar arithmetic, free beside the MFMAs) plus a 32-bit
    // lane offset that is fixed for the whole kernel: up to three per operand, by q mod 2 (along k) or q mod 3.
    // K-tiles beyond the last one (the pipeline asks for two ahead) repeat the last: in bounds and never read.
    auto lane_offset = [&](auto layout, auto extent, int64_t ld, int q) -> uint32_t {
        constexpr int LAY = decltype(layout)::value, EXT = decltype(extent)::value;
        if constexpr (LAY == kKContig) {
            return (uint32_t)(((lane >> 3) * ld + (((lane & 7) ^ ((4 * (q & 1) + (lane >> 4)) & 7)) << 2)) << 2);
        } else {
            const int pos = (1024 * q) % (4 * EXT) + 16 * lane;
            return (uint32_t)((pos / (4 * EXT)) * ld * 4 + pos % (4 * EXT));
        }
    };
    using LayA = std::integral_constant<int, ALAY>;
    using LayB = std::integral_constant<int, BLAY>;
    using ExtA = std::integral_constant<int, BM>;
    using ExtB = std::integral_constant<int, BN>;
    const uint32_t a_off[3] = {lane_offset(LayA{}, ExtA{}, g.lda, 0), lane_offset(LayA{}, ExtA{}, g.lda, 1), lane_offset(LayA{}, ExtA{}, g.lda, 2)};
    const uint32_t b_off[3] = {lane_offset(LayB{}, ExtB{}, g.ldb, 0), lane_offset(LayB{}, ExtB{}, g.ldb, 1), lane_offset(LayB{}, ExtB{}, g.ldb, 2)};
    // The loads of a K-tile in issue order: A's and B's alternate while both last.  -> operand (0 A, 1 B) and q
    auto which = [](int idx, int &operand, int &q) {
        constexpr int kBoth = 2 * (kLoadsA < kLoadsB ? kLoadsA : kLoadsB);
        if (idx < kBoth) operand = idx & 1, q = idx >> 1;
        else operand = kLoadsA < kLoadsB ? 1 : 0, q = idx - kBoth / 2;
    };
    // A load is issued by hand in two steps: M0 <- its LDS address, then, at least one instruction later (M0 needs a
    // wait state before a load reads it), the load in its scalar-base form.
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(LDS_PTR char *)lds);
    auto load_m0 = [&](int stage, int idx) {
        int operand, q;
        which(idx, operand, q);
        // (worked out anew each time, like the bases below: see there)
        uint32_t dst = lds0 + wave * ((operand ? kLoadsB : kLoadsA) * 1024);
        asm volatile("" : "+s"(dst));
        dst += stage * kStageBytes + operand * kBytesA + q * 1024;
        asm volatile("s_mov_b32 m0, %0" ::"s"(dst) : "m0");
    };
    auto dma = [&](auto layout, auto extent, const float *__restrict__ P, int64_t ld, int origin, const uint32_t (&off)[3], int q, int t) {
        constexpr int LAY = decltype(layout)::value, EXT = decltype(extent)::value;
        const int tc = t < nk ? t : nk - 1;
        // The base is worked out anew for every load (a handful of scalar instructions): kept across the loop, the
        // bases of all loads would not fit the scalar registers, and a spilled one would come back through a lane
        // read right in front of a hand-issued load, which the compiler does not know to keep apart.  The zero
        // below is opaque to it, so nothing that contains it is loop-invariant.
        int zero = 0;
        asm volatile("" : "+s"(zero));
        const float *row;       // uniform
        if constexpr (LAY == kKContig) row = P + (int64_t)(origin + wave * (EXT / 4) + 8 * q + zero) * ld + tc * kBK;
        else row = P + (int64_t)(tc * kBK + (wave * (EXT / 32) + q) * 256 / EXT) * ld + origin;
        const int variant = LAY == kKContig ? q & 1 : EXT == 192 ? q % 3 : 0;      // which of the operand's lane offsets
        asm volatile("global_load_lds_dwordx4 %0, %1" ::"v"(off[variant]), "s"(row) : "memory");
    };
    auto load_go = [&](int idx, int t) {
        int operand, q;
        which(idx, operand, q);
        if (operand) dma(LayB{}, ExtB{}, B, g.ldb, n0, b_off, q, t);
        else dma(LayA{}, ExtA{}, A, g.lda, m0, a_off, q, t);
    };
    auto load = [&](int stage, int idx, int t) {    // outside the MFMA loop
        load_m0(stage, idx);
        asm volatile("s_nop 0" ::: "memory");
        load_go(idx, t);
    };

    // Fragments of chunk c (8 k): the lane with row / column x = offset + 32 block + lane % 32 holds
    // k = 8 c + 4 (lane / 32) + s for the four steps s of the chunk -- one 16-byte read along k, four 4-byte
    // reads along m / n.
    float fa[2][WM][4], fb[2][WN][4];       // [register buffer][block][step]
    constexpr int kReadsA = ALAY == kKContig ? WM : 4 * WM, kReadsB = BLAY == kKContig ? WN : 4 * WN;
    constexpr int kReads = kReadsA + kReadsB;
    // A chunk has a slot behind each MFMA.  The larger shapes put one fragment read behind an MFMA and the loads behind
    // every second MFMA at the end of chunk 3; tiles with a side of 64 have 4 to 8 MFMAs per chunk, so they take up to
    // two reads behind one MFMA and a load behind every MFMA (a 64-cycle MFMA still covers them).
    constexpr int kReadsPerSlot = (kReads + kMfmas - 1) / kMfmas, kLoadStride = 2 * kLoads <= kMfmas ? 2 : 1;
    static_assert(kReadsPerSlot <= 2 && kLoadStride * kLoads <= kMfmas, "slots of a chunk");
    auto fragment = [&](auto layout, auto extent, auto blocks, const char *st, int offset, int c, auto &f, int idx) {
        constexpr int LAY = decltype(layout)::value, EXT = decltype(extent)::value, W = decltype(blocks)::value;
        if constexpr (LAY == kKContig) {
            const int b = idx;
            const f32x4 v = *reinterpret_cast<const f32x4 *>(st + (offset + 32 * b + li) * 128 + (((2 * c + lh) ^ ((li >> 1) & 7)) << 4));
#pragma unroll
            for (int s = 0; s < 4; ++s) f[b][s] = v[s];
        } else {
            const int b = idx % W, s = idx / W;
            const int k = 8 * c + 4 * lh + s, x = offset + 32 * b + li;
            f[b][s] = *reinterpret_cast<const float *>(st + k * (4 * EXT) + 4 * x);
        }
    };
    auto read = [&](int stage, int c, int buf, int idx) {   // idx 0 .. kReads - 1
        const char *st = lds + stage * kStageBytes;
        if (idx < kReadsA) fragment(LayA{}, ExtA{}, std::integral_constant<int, WM>{}, st, wm0, c, fa[buf], idx);
        else fragment(LayB{}, ExtB{}, std::integral_constant<int, WN>{}, st + kBytesA, wn0, c, fb[buf], idx - kReadsA);
    };

    f32x16 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
            asm volatile("" : "+a"(acc[i][j]));
        }

    // K-tiles 0 and 1 into stages 0 and 1, then the first fragments
#pragma unroll
    for (int idx = 0; idx < kLoads; ++idx) load(0, idx, 0);
#pragma unroll
    for (int idx = 0; idx < kLoads; ++idx) load(1, idx, 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    FENCE();
#pragma unroll
    for (int idx = 0; idx < kReads; ++idx) read(0, 0, 0, idx);
    FENCE();

    auto k_tile = [&](auto parity, int t) {
        constexpr int X = decltype(parity)::value, Y = 1 - X;
        constexpr int kFirstLoadSlot = kMfmas - kLoadStride * kLoads;         // the loads sit behind every second MFMA (every MFMA) at the end of chunk 3
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int cur = c & 1, nxt = cur ^ 1;
#pragma unroll
            for (int m = 0; m < kMfmas; ++m) {
                const int s = m / (WM * WN), i = (m / WN) % WM, j = m % WN;
                const bool loads = c == 3 && m >= kFirstLoadSlot && (m - kFirstLoadSlot) % kLoadStride == 0;
                if (loads) load_m0(X, (m - kFirstLoadSlot) / kLoadStride);
                {
                    const float av = fa[cur][i][s], bv = fb[cur][j][s];
                    asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(av), "v"(bv));
                }
                if (loads) load_go((m - kFirstLoadSlot) / kLoadStride, t + 2);
#pragma unroll
                for (int r = kReadsPerSlot * m; r < kReadsPerSlot * (m + 1) && r < kReads; ++r) {
                    if (c < 3) read(X, c + 1, nxt, r);
                    else read(Y, 0, nxt, r);
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

    // The rest of K when K is not whole K-tiles (it is a multiple of 4, so a piece lies inside K or beyond it): one
    // more K-tile whose pieces beyond K come from a zero piece.  It runs outside the pipeline, once per tile of C: its
    // loads (one address per lane, through the compiler's builtin) are waited for, then its chunks run with their
    // fragment reads in front of them.  Nothing of it may be kept in registers across the loop (the 256 x 256 tile has
    // none to spare): the lane's number is read again from the hardware here and in the epilogue.
    const int k_rest = g.K - nk * kBK;
    if (k_rest > 0) {
        // (the lane's number is taken afresh from the hardware: nothing of this step is to be worked out, and kept in
        // registers, ahead of the loop)
        int ln = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        asm volatile("" : "+v"(ln));
        auto tail_src = [&](auto layout, auto extent, const float *__restrict__ P, int64_t ld, int origin, int q) -> const float * {
            constexpr int LAY = decltype(layout)::value, EXT = decltype(extent)::value;
            if constexpr (LAY == kKContig) {
                const int piece = (ln & 7) ^ ((4 * (q & 1) + (ln >> 4)) & 7);
                const int row = origin + wave * (EXT / 4) + 8 * q + (ln >> 3);
                return 4 * piece < k_rest ? P + (int64_t)row * ld + nk * kBK + 4 * piece : kZeroPiece;
            } else {
                const int pos = (1024 * q) % (4 * EXT) + 16 * ln;
                const int k_row = (wave * (EXT / 32) + q) * 256 / EXT + pos / (4 * EXT);
                return k_row < k_rest ? P + (int64_t)(nk * kBK + k_row) * ld + origin + (pos % (4 * EXT)) / 4 : kZeroPiece;
            }
        };
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();       // every load has landed and every wavefront is done with both stages
        FENCE();
#pragma unroll
        for (int idx = 0; idx < kLoads; ++idx) {
            int operand, q;
            which(idx, operand, q);
            char *dst = lds + operand * kBytesA + (wave * (operand ? kLoadsB : kLoadsA) + q) * 1024;       // stage 0
            const float *src = operand ? tail_src(LayB{}, ExtB{}, B, g.ldb, n0, q) : tail_src(LayA{}, ExtA{}, A, g.lda, m0, q);
            __builtin_amdgcn_global_load_lds((const GLOBAL_PTR void *)src, (LDS_PTR void *)dst, 16, 0, 0);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        FENCE();
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (8 * c < k_rest) {
#pragma unroll
                for (int idx = 0; idx < kReads; ++idx) read(0, c, 0, idx);
                FENCE();
#pragma unroll
                for (int m = 0; m < kMfmas; ++m) {
                    const int s = m / (WM * WN), i = (m / WN) % WM, j = m % WN;
                    const float av = fa[0][i][s], bv = fb[0][j][s];
                    asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(av), "v"(bv));
                }
                FENCE();
            }
        }
    }

    // Every global->LDS load has landed before the workgroup gives up its LDS, and the last MFMAs (64 cycles each,
    // unknown to the compiler as such) have written their accumulators before these are read.
    asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
    // (the lane's number is taken afresh from the hardware, so that no store address is kept in a register across the loop)
    int lane_e = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    asm volatile("" : "+v"(lane_e));
    const int li_e = lane_e & 31, lh_e = lane_e >> 5;
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int col = n0 + wn0 + j * 32 + li_e;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm0 + i * 32 + (r / 4) * 8 + lh_e * 4 + (r % 4);
                g.C[(int64_t)row * g.ldc + col] = acc[i][j][r];
            }
            FENCE();
        }
}

template <int WM, int WN, int ALAY, int BLAY>
hipError_t launch_main(const GemmArgs &a, hipStream_t s)
{
    constexpr int kLdsBytes = 2 * (64 * WM + 64 * WN) * kBK * 4;
    auto kern = gemm_f32_main_kernel<WM, WN, ALAY, BLAY>;
    static std::atomic<uint64_t> configured{0};
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), kLdsBytes, configured);
    if (e != hipSuccess) return e;
    const int tiles_m = (a.M + 64 * WM - 1) / (64 * WM), tiles_n = (a.N + 64 * WN - 1) / (64 * WN);
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n * a.k_slices)), dim3(kThreads), kLdsBytes, s, a, tiles_m, tiles_n);
    return hipGetLastError();
}

template <int WM, int WN>
hipError_t launch_shape(int a_lay, int b_lay, const GemmArgs &a, hipStream_t s)
{
    if (a_lay == kKContig) return b_lay == kKContig ? launch_main<WM, WN, kKContig, kKContig>(a, s) : launch_main<WM, WN, kKContig, kMnContig>(a, s);
    return b_lay == kKContig ? launch_main<WM, WN, kMnContig, kKContig>(a, s) : launch_main<WM, WN, kMnContig, kMnContig>(a, s);
}

// in the order of the candidate numbers, which is the order the shapes were added in
constexpr int kShapeM[kF32MainShapes] = {256, 192, 128, 256, 192, 128, 256, 192, 128, 64, 128, 64}, kShapeN[kF32MainShapes] = {256, 256, 256, 128, 128, 128, 192, 192, 192, 64, 64, 128};

}  // namespace

int f32_main_tile_m(int shape) { return kShapeM[shape]; }
int f32_main_tile_n(int shape) { return kShapeN[shape]; }

// <blocks of 32 rows per wavefront, blocks of 32 columns, A layout, B layout> with 0 = contiguous along k, 1 = along
// m / n; as a profiler trace prints the kernel
const char *f32_main_kernel_name(int shape, int a_lay, int b_lay)
{
    struct Names {
        char text[kF32MainShapes][2][2][40];
        Names()
        {
            for (int sh = 0; sh < kF32MainShapes; ++sh)
                for (int a = 0; a < 2; ++a)
                    for (int b = 0; b < 2; ++b)
                        snprintf(text[sh][a][b], sizeof text[sh][a][b], "gemm_f32_main_kernel<%d, %d, %d, %d>", kShapeM[sh] / 64, kShapeN[sh] / 64, a, b);
        }
    };
    static const Names names;
    return names.text[shape][a_lay][b_lay];
}

// Whole unchecked tiles of 16-byte pieces: a matrix at least one tile high and wide (a ragged last tile is shifted
// back into it), at least one K-tile of 32 and K a multiple of 4, 16-byte aligned bases and rows,
// for an operand that is contiguous along
// m (n) M (N) a multiple of 4 so that a shifted tile still starts on a piece; leading dimensions below 2^24 elements,
// because a lane's offset from its load's uniform base (up to 7 rows and 28 elements along k, up to 2 k-rows along
// m / n) is a 32-bit number of bytes.
bool f32_main_fits(int shape, int a_lay, int b_lay, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb)
{
    if (shape < 0 || shape >= kF32MainShapes) return false;
    const int bm = kShapeM[shape], bn = kShapeN[shape];
    const bool aligned = ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 15u) == 0 && lda % 4 == 0 && ldb % 4 == 0;
    return aligned && lda < kF32MaxLdUnchecked && ldb < kF32MaxLdUnchecked && M >= bm && N >= bn && K >= kBK && K % 4 == 0 && (a_lay == kKContig || M % 4 == 0) &&
           (b_lay == kKContig || N % 4 == 0) && ((M + bm - 1) / bm) * ((N + bn - 1) / bn) < ((int64_t)1 << 31);
}

// K may be cut into `slices` whole numbers of K-tiles if the last slice still has a whole K-tile
bool f32_main_slices_fit(int64_t K, int slices)
{
    return slices >= 1 && K < ((int64_t)1 << 31) && (int64_t)(slices - 1) * main_slice_length((int)K, slices) + kBK <= K;
}

// requires f32_main_fits(...) and f32_main_slices_fit(a.K, a.k_slices); with slices, a.C is the workspace and a.ldc = a.N
hipError_t launch_f32_main(int shape, int a_lay, int b_lay, const GemmArgs &a, hipStream_t s)
{
    if (!f32_main_fits(shape, a_lay, b_lay, a.M, a.N, a.K, a.A, a.lda, a.B, a.ldb) || !f32_main_slices_fit(a.K, a.k_slices)) return hipErrorInvalidValue;
    if (((a.M + kShapeM[shape] - 1) / kShapeM[shape]) * (int64_t)((a.N + kShapeN[shape] - 1) / kShapeN[shape]) * a.k_slices >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    switch (shape) {
    case 0: return launch_shape<4, 4>(a_lay, b_lay, a, s);
    case 1: return launch_shape<3, 4>(a_lay, b_lay, a, s);
    case 2: return launch_shape<2, 4>(a_lay, b_lay, a, s);
    case 3: return launch_shape<4, 2>(a_lay, b_lay, a, s);
    case 4: return launch_shape<3, 2>(a_lay, b_lay, a, s);
    case 5: return launch_shape<2, 2>(a_lay, b_lay, a, s);
    case 6: return launch_shape<4, 3>(a_lay, b_lay, a, s);
    case 7: return launch_shape<3, 3>(a_lay, b_lay, a, s);
    case 8: return launch_shape<2, 3>(a_lay, b_lay, a, s);
    case 9: return launch_shape<1, 1>(a_lay, b_lay, a, s);
    case 10: return launch_shape<2, 1>(a_lay, b_lay, a, s);
    default: return launch_shape<1, 2>(a_lay, b_lay, a, s);
    }
}

}  // namespace fsrgemm
