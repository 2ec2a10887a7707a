// Main bf16 kernel for large, aligned problems: C[M x N] = A . B, fp32
// accumulate and output -- the Task 2 product at matrix-core input precision.
// Either operand may be contiguous along k (a row-major A, a column-major B:
// the tile's rows are 128 bytes of 64 k) or along m / n (a transposed A, a
// row-major B: the tile is kept as k-rows, 128 bytes of 64 m or n each); LDS keeps the
// memory order and the fragment reads do the rest (see "Fragments" below).
//
// Shape of the computation (for the 256 x 256 tile; "Tile shapes" below)
//   workgroup  : 256 lanes = 4 wavefronts, one per SIMD, 256 x 256 tile of C
//   wavefront  : 128 x 128 of that tile = 8 x 8 blocks of V_MFMA_F32_16X16X32_BF16,
//                256 accumulator registers (the whole AccVGPR file)
//   K-tile     : 64 elements = one 128-byte row per tile row, 2 MFMA k-steps of 32
//   LDS        : two stages of (A 32 KB + B 32 KB); stage t%2 is read while
//                stage (t+1)%2 is filled by direct global->LDS loads
//
// Why the 16x16x32 instruction: this part runs bf16 matrix work against its
// power limit, not its issue rate.  Per flop the 16x16x32 form moves half the
// accumulator data of the 32x32x16 form through the register file; a
// register-only loop on random operands sustains about 2.0 PFLOP/s with it
// against 1.7-1.8 with 32x32x16 (both reach 2.4 on zeros).
//
// A large tile is what keeps the path inside the L2 bandwidth: each K-tile
// moves 64 KB into the workgroup for 33.5 MFLOP.  With one wavefront per SIMD
// nothing else can fill an issue bubble, and a 16-cycle MFMA leaves room for
// about three other instructions, so the loop is an explicit schedule, fenced
// slot by slot: 128 MFMAs per K-tile carry 32 LDS fragment reads, 16
// global->LDS loads, one prefetch touch and a handful of address updates, never
// more than two of them behind one MFMA.
//
// The loads are issued by hand.  Through the compiler's builtin a load costs a
// 64-bit vector add, an M0 write, a wait state and the load itself -- more than
// a slot holds.  Here the address is a scalar row-group base (16 of them, fixed
// for the tile) plus a 32-bit lane offset that also carries the K position (4
// registers, advanced once per K-tile); M0 (the LDS destination) is written
// one slot ahead, so the MFMA in between is the wait state M0 needs.
//
// The MFMAs are inline assembly for one reason: written with the builtin, the
// register allocator permutes the 64 four-register accumulators across the
// loop's back edge and fills the loop with hundreds of accumulator moves.  With
// "+a" operands every block stays where it is.  The compiler cannot see that
// these statements are MFMAs, so the hazards it would cover are kept away by
// construction: a block's two MFMAs of a K-tile follow each other directly with
// the same accumulator registers as result and addend (the one dependence the
// matrix core resolves itself; see ChainPlan below for why they are paired),
// the block is touched again only a K-tile later, and the epilogue starts
// behind explicit wait states.
//
// Per K-tile t of parity P (stage X = P holds t, Y = 1 - P receives t+1), all
// fragments of t being in registers or on their way when it starts:
//   first half : MFMAs; the last fragment reads of X (into registers K-tile t-1
//              has freed); the late loads of K-tile t+1 into Y; the prefetch touch
//   barrier  : all loads but the touch have landed (Y complete), every
//              wavefront has all fragments of X in registers
//   second half : MFMAs; fragment reads of Y (K-tile t+1) into the registers this
//              K-tile has freed; the early loads of K-tile t+2 into X
// A load thus has at least half a K-tile (about 1000 cycles) to arrive: enough
// for an L2 hit, not for a first touch that has to come over the fabric.  Each
// workgroup therefore also touches, three K-tiles ahead, its share of the
// operand rows that the workgroups running beside it on the same XCD read as
// well (with the tile order of tile_coords, 4 neighbours share an A panel and 8
// share a B panel): one 4-byte global->LDS load per wavefront whose lanes each
// hit a different 128-byte line.  The data is discarded; the lines are then in
// L2 when the real loads of all sharers arrive.
//
// Fragments.  The MFMA wants, per lane, 8 consecutive k of row l % 16 at
// k-offset 8 (l / 16).  For an operand contiguous along k that is one 16-byte
// LDS read: rows are 128 bytes, unpadded, 16-byte chunk c of row r stored at
// chunk position c ^ ((r >> 1) & 7), so that a 16-lane group (16 rows, one
// chunk) touches all 64 banks once.  For an operand contiguous along m / n it
// is two transposing reads (DS_READ_B64_TR_B16): within a 16-lane group, lane
// i receives element i % 4 of the 8 bytes that lanes i / 4, 4 + i / 4,
// 8 + i / 4 and 12 + i / 4 point at.  Lane s therefore points at k-row
// k0 + s / 4, rows 4 (s % 4) .. + 3 of the block, and lane i ends up with
// k0 .. k0 + 3 of row i; k0 = 8 (l / 16) for the first read, + 4 for the second.
// Such a tile is kept in LDS as sub-tiles of 64 rows (4 blocks), whatever
// its side (256, 192 or 128: a k-row of 384 bytes would fit no power-of-two
// scheme): a load places 8 k-rows of 128 bytes of one sub-tile, 16-byte chunk
// c of k-row k at c ^ f(k), f(k) = 2 ((k / 2) % 2) + 4 ((k / 8) % 2).  The 32
// lanes one pass of the read serves (4 + 4 k-rows, 32 bytes each; odd k-rows
// start 128 bytes into the 256 the banks span) then cover all 64 banks once.
// The blocks of a sub-tile differ by an XOR in address bits 5-6, so a lane
// keeps one address per block (one register per block and such operand) and
// reaches k-step, half and stage through immediate offsets.  (Whole k-rows
// of 512 and 256 bytes with their own swizzle, the first design for sides of
// 256 and 128, ran level with this on every size tried and were dropped.)
//
// Tile shapes.  A launch lasts as long as the compute unit with the most tiles, so a problem whose 256 x 256
// tiles do not fill whole rounds of the compute units is better off with a tile that does: the kernel is a
// template over the blocks per wavefront, IM x JN of 16 x 16 (tile 32 IM x 32 JN), built for sides of 256, 192
// and 128.  (A 128 x 128 tile asks the L2 for more bytes per cycle than a compute unit gets; it is there for problems
// too small to give every compute unit a larger tile, where two such workgroups share a unit.)
// Everything scales: IM + JN loads per wavefront and K-tile, IM + JN fragment reads and IM JN MFMAs per
// k-step.  The 128 x 128 tile has 16 MFMAs per half of
// a K-tile: its loads sit behind every third MFMA and its fragment reads behind consecutive ones.
//
// Rest of K.  When K is not whole K-tiles (it is a multiple of 8, so a 16-byte piece lies inside K or beyond
// it), one more K-tile follows the pipeline, once per tile of C: its loads take an address per lane through the
// compiler's builtin, pieces beyond K come from a zero piece in device memory, the loads are waited for, then
// the k-steps that contain k < K run with their fragment reads in front.
#include <stdio.h>

#include <type_traits>
#include <utility>

#include "launchers.hpp"

namespace fsrgemm {
namespace {

#define FSR_AS3 __attribute__((address_space(3)))

// M0 is on the clobber lists below on purpose (the loads take their LDS address from it); clang warns
// that it is a reserved register.  Nothing the compiler emits for this kernel uses M0.
#pragma clang diagnostic ignored "-Winline-asm"

constexpr int kBK = 64;

// k per slice when K is cut into `slices`: a whole number of K-tiles, the last slice takes what is left
__host__ __device__ constexpr int bf16_main_slice_length(int K, int slices) { return ((K + kBK - 1) / kBK + slices - 1) / slices * kBK; }
constexpr int kScratchBytes = 1024;             // landing zone of the prefetch touches (256 B per wavefront)
constexpr int kThreads = 256;
constexpr int kLate = 4;         // loads of K-tile t+1 issued in k-step 0 of K-tile t; the others earlier, in k-step 1 of t-1
// a load behind every fourth MFMA (slots 2, 6, ...): denser loads stall the matrix pipe; every third where a half has
// fewer than 32 slots (tiles with both sides below 256)
constexpr int load_every(int mfmas_per_half) { return mfmas_per_half >= 32 ? 4 : 3; }

// where the loads of the last, partial K-tile fetch the pieces that lie beyond K
__device__ __attribute__((aligned(16))) const uint16_t kZeroPiece[8] = {0, 0, 0, 0, 0, 0, 0, 0};

#define FSR_AS1 __attribute__((address_space(1)))

// Order of the MFMAs and of the fragment reads of one K-tile.
//
// Every 16 x 16 block of the wavefront's part takes its two MFMAs of a K-tile (k-steps 0 and 1) directly one
// after the other: the second then takes the first one's result as its addend without that result passing through
// the register file, which draws measurably less power (register-only loops on random operands: 2.03 PFLOP/s with
// a block's MFMAs 64 apart, 2.15 in pairs), and power is what bounds this kernel.  A K-tile therefore needs all
// 2 (IM + JN) fragments of both k-steps, and each fragment register is filled again with the next K-tile's
// fragment once its last MFMA of this K-tile has been issued.  For that to leave every read time, the walk over
// the blocks alternates: K-tiles of stage 0 go row by row (fragment a_i is free after row i, the b_j only in the
// last row), K-tiles of stage 1 column by column (b_j free after column j) -- the fragments that become free last
// in one walk are those the other walk needs last.  "Slot" s = 2 p + kk is the MFMA of k-step kk on the p-th
// block of the walk; the barrier sits after slot H - 1 (H = IM JN, half the slots), and a K-tile's fragments are
// read between the barrier of the K-tile before and its own barrier, the only time its stage is complete and not
// yet being overwritten.  The plan below places these reads at compile time: at every slot that may carry a read
// (not those behind which a global load or the touch is issued, at most every second slot) the free register
// whose fragment is needed first is filled; the static_asserts check that every read has a lead of kMinLead slots
// on its first use and that the last reads are issued well ahead of the barrier that waits for them.
template <int IM, int JN, int LATE, int EARLY, int LOAD_EVERY, int TOUCH_SLOT>
struct ChainPlan {
    static constexpr int H = IM * JN, S = 2 * H, NF = 2 * (IM + JN);
    static constexpr int kMinLead = 6, kReadGap = H >= 32 ? 2 : 1;
    // fragment f < NF: k-step f / (IM + JN); r = f % (IM + JN) < IM is a_r, else b_(r - IM)
    static constexpr int kk_of(int f) { return f / (IM + JN); }
    static constexpr bool is_a(int f) { return f % (IM + JN) < IM; }
    static constexpr int idx_of(int f) { return is_a(f) ? f % (IM + JN) : f % (IM + JN) - IM; }
    // walk 0: row by row, walk 1: column by column; p-th block
    static constexpr int blk_i(int walk, int p) { return walk == 0 ? p / JN : p % IM; }
    static constexpr int blk_j(int walk, int p) { return walk == 0 ? p % JN : p / IM; }
    static constexpr int first_slot(int walk, int f)
    {
        const int x = idx_of(f), p = walk == 0 ? (is_a(f) ? x * JN : x) : (is_a(f) ? x : x * IM);
        return 2 * p + kk_of(f);
    }
    static constexpr int last_slot(int walk, int f)
    {
        const int x = idx_of(f), p = walk == 0 ? (is_a(f) ? x * JN + JN - 1 : (IM - 1) * JN + x) : (is_a(f) ? (JN - 1) * IM + x : x * IM + IM - 1);
        return 2 * p + kk_of(f);
    }
    // may a fragment read follow the MFMA of slot m of half h?  Not where a global load or the touch follows it.
    static constexpr bool read_slot(int h, int m)
    {
        const int c = m / LOAD_EVERY;
        const bool has_load = h == 1 ? c < EARLY : c < LATE;
        if (m % LOAD_EVERY == 2 && has_load) return false;
        if (h == 0 && m == TOUCH_SLOT + 1) return false;
        return true;
    }
    struct Plan {
        int frag[S];        // [u - H] for u in [H, H + S): the fragment read behind slot u of the timeline below, or -1
        int min_lead, last_read;
        bool complete;
    };
    // Reads that take the fragments from a K-tile walked as `from` to the next (walked the other way).  Timeline u:
    // slots of the first K-tile are u = 0 .. S - 1, of the second S + 0 ..; reads may be issued for u in [H, H + S).
    static constexpr Plan make(int from)
    {
        Plan pl{};
        for (int u = 0; u < S; ++u) pl.frag[u] = -1;
        bool done[NF] = {};
        int placed = 0, last = -kReadGap;
        pl.min_lead = S;
        pl.last_read = 0;
        for (int u = H; u < H + S; ++u) {
            if (!read_slot((u / H) % 2, u % H) || u - last < kReadGap) continue;
            int best = -1, best_need = 0;
            for (int f = 0; f < NF; ++f) {
                if (done[f] || last_slot(from, f) + 1 > u) continue;
                const int need = S + first_slot(1 - from, f);
                if (best < 0 || need < best_need) best = f, best_need = need;
            }
            if (best < 0) continue;
            done[best] = true;
            pl.frag[u - H] = best;
            last = u;
            ++placed;
            if (best_need - u < pl.min_lead) pl.min_lead = best_need - u;
            pl.last_read = u;
        }
        pl.complete = placed == NF;
        return pl;
    }
    static constexpr Plan kPlan[2] = {make(0), make(1)};
    static_assert(kPlan[0].complete && kPlan[1].complete, "every fragment register is filled again");
    static_assert(kPlan[0].min_lead >= kMinLead && kPlan[1].min_lead >= kMinLead, "a read is issued kMinLead MFMAs ahead of its first use");
    static_assert(kPlan[0].last_read + kMinLead <= H + S && kPlan[1].last_read + kMinLead <= H + S, "the last reads are issued well ahead of the barrier");
};

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

template <int I>
using Int = std::integral_constant<int, I>;

template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(Int<Is>{}), ...);
}
// f(Int<0>{}), ..., f(Int<N-1>{}): a loop whose index is a compile-time constant in the body
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// chunk swizzle of k-row k of an operand that is contiguous along m / n (in units of 16-byte chunks)
__device__ __forceinline__ int kswz(int k) { return (((k >> 1) & 1) | (((k >> 3) & 1) << 1)) << 1; }

template <int IM, int JN, int ALAY, int BLAY>
__global__ __launch_bounds__(kThreads) void gemm_bf16_main_kernel(GemmArgs g, int tiles_m, int tiles_n)
{
    constexpr bool AMC = ALAY == kMnContig, BMC = BLAY == kMnContig;
    constexpr int kBM = 32 * IM, kBN = 32 * JN;
    constexpr int kTileA = kBM * kBK * 2, kTileB = kBN * kBK * 2;       // operand tiles: 128 bytes per row
    constexpr int kStageBytes = kTileA + kTileB;
    constexpr int kLoadsA = IM, kLoadsB = JN, kLoads = IM + JN;        // 1 KB each, per wavefront and K-tile
    constexpr int kMfmas = IM * JN;                                    // per k-step
    constexpr int kReads = IM + JN;                                    // fragment reads per k-step
    constexpr int kEarly = kLoads - kLate;
    constexpr int kLoadEvery = load_every(kMfmas);
    // K-tiles between a prefetch touch and the loads it serves: with 64 MFMAs per k-step 2 is too late, 4 and more
    // let touched lines be evicted before use (more fabric reads, same time); shorter K-tiles look one further ahead
    constexpr int kTouchAhead = kMfmas == 64 ? 3 : 4;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    // K slices (a call with a workspace): workgroup ids beyond the first tiles_m * tiles_n belong to further slices.
    // Slice s is the product over k in [s per, s per + its length) with per a whole number of K-tiles, written to the
    // s-th M x N block behind g.C (the workspace, tightly packed: the launcher sets ldc = N): for the rest of the kernel
    // it is simply a product of its own, on operands shifted along k.
    int pid = blockIdx.x;
    if (g.k_slices > 1) {
        const int tiles = tiles_m * tiles_n, slice = pid / tiles;
        pid -= slice * tiles;
        const int per = bf16_main_slice_length(g.K, g.k_slices), k0 = slice * per;
        g.A = static_cast<const uint16_t *>(g.A) + (AMC ? (int64_t)k0 * g.lda : (int64_t)k0);
        g.B = static_cast<const uint16_t *>(g.B) + (BMC ? (int64_t)k0 * g.ldb : (int64_t)k0);
        g.K = min(per, g.K - k0);
        g.C += (int64_t)slice * g.slice_stride;
    }
    int tile_m, tile_n;
    tile_coords(pid, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_origin(tile_m, kBM, g.M), n0 = tile_origin(tile_n, kBN, g.N);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave >> 1) * (16 * IM), wn0 = (wave & 1) * (16 * JN);
    const int l16 = lane & 15, lq = lane >> 4;
    const int nk = g.K / kBK;
    const uint16_t *A = static_cast<const uint16_t *>(g.A);
    const uint16_t *B = static_cast<const uint16_t *>(g.B);

    // Global -> LDS.  A load instruction moves 64 x 16 bytes to 1 KB of contiguous LDS; a wavefront fills its
    // quarter of each operand tile (8 IM KB of A, 8 JN KB of B) with IM + JN loads (index q < IM for A, IM + q for B).
    //   contiguous along k    : 8 tile rows per load: rows 8 IM w + 8 q + lane / 8 (8 JN w + .. for B); the lane fetches
    //                           the chunk that belongs at its position, (lane % 8) ^ ((row >> 1) & 7), and
    //                           ((8 IM w + 8 q + lane / 8) >> 1) & 7 = 4 (q & 1) + (lane / 8 >> 1) for even IM: one lane
    //                           offset for even q, one for odd q.  The lane offsets also carry the K position.
    //   contiguous along m / n: 8 k-rows of one 64-row sub-tile per load, 128 bytes each: sub-tile q / 2, k-rows
    //                           16 w + 8 (q & 1) + lane / 8, chunk (lane % 8) ^ kswz(k-row), and of the k-row only
    //                           (k / 2) % 2 = (lane / 16) % 2 and (k / 8) % 2 = q & 1 enter kswz: one lane offset for
    //                           even q, one for odd q.  The K position is carried by the scalar row bases.
    const int lrow = lane >> 3, lpos = lane & 7;
    const int sw_even = (lrow >> 1) & 3, sw_odd = sw_even ^ 4;
    uint32_t voff_a[2], voff_b[2];      // bytes
#pragma unroll
    for (int v = 0; v < 2; ++v) {
        const int kc_chunk = lpos ^ (v ? sw_odd : sw_even), mn_chunk = lpos ^ kswz(lrow + 8 * v);
        voff_a[v] = AMC ? (uint32_t)(lrow * g.lda * 2 + mn_chunk * 16) : (uint32_t)(lrow * g.lda + kc_chunk * 8) * 2u;
        voff_b[v] = BMC ? (uint32_t)(lrow * g.ldb * 2 + mn_chunk * 16) : (uint32_t)(lrow * g.ldb + kc_chunk * 8) * 2u;
    }
    const char *rbase[kLoads];      // row-group bases: uniform; fixed for the tile unless they carry the K position
#pragma unroll
    for (int q = 0; q < kLoadsA; ++q)
        rbase[q] = AMC ? reinterpret_cast<const char *>(A + (int64_t)(wave * 16 + (q & 1) * 8) * g.lda + m0 + 64 * (q >> 1))
                       : reinterpret_cast<const char *>(A + (int64_t)(m0 + wave * (8 * IM) + q * 8) * g.lda);
#pragma unroll
    for (int q = 0; q < kLoadsB; ++q)
        rbase[kLoadsA + q] = BMC ? reinterpret_cast<const char *>(B + (int64_t)(wave * 16 + (q & 1) * 8) * g.ldb + n0 + 64 * (q >> 1))
                                 : reinterpret_cast<const char *>(B + (int64_t)(n0 + wave * (8 * JN) + q * 8) * g.ldb);
    const int64_t kstep_a = 64 * g.lda * 2, kstep_b = 64 * g.ldb * 2;       // one K-tile of k-rows, in bytes
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(FSR_AS3 char *)smem);
    const uint32_t wave_lds_a = lds0 + wave * (kLoadsA * 1024), wave_lds_b = lds0 + kTileA + wave * (kLoadsB * 1024);
    // M0 <- LDS address of load `idx` in `stage`; at least one instruction must follow before the load
    auto load_m0 = [&](auto stage, auto idx) {
        constexpr int I = decltype(idx)::value;
        constexpr int kOff = decltype(stage)::value * kStageBytes + (I < kLoadsA ? I : I - kLoadsA) * 1024;
        const uint32_t w = I < kLoadsA ? wave_lds_a : wave_lds_b;
        asm volatile("s_add_u32 m0, %0, %1" ::"s"(w), "n"(kOff) : "m0", "scc");
    };
    bool more = 1 < nk;     // the K-tile after the one now being loaded lies inside K (else the last one is loaded again)
    auto load_go = [&](auto idx) {
        constexpr int I = decltype(idx)::value, q = I < kLoadsA ? I : I - kLoadsA;
        constexpr bool mc = I < kLoadsA ? AMC : BMC;
        const uint32_t vo = I < kLoadsA ? voff_a[q & 1] : voff_b[q & 1];
        const char *rb = rbase[I];
        asm volatile("global_load_lds_dwordx4 %0, %1" ::"v"(vo), "s"(rb) : "memory");
        if constexpr (mc) rbase[I] += more ? (I < kLoadsA ? kstep_a : kstep_b) : 0;      // its next use is the next K-tile
    };
    // after the last load of a K-tile: the following loads fetch K-tile `next`; past the end they stay on
    // the last K-tile, whose data then lands once more in a stage that is never read again
    auto advance = [&](int next) {
        more = next + 1 < nk;
        const uint32_t step = next < nk ? (uint32_t)(kBK * 2) : 0u;
        if (!AMC) voff_a[0] += step, voff_a[1] += step;
        if (!BMC) voff_b[0] += step, voff_b[1] += step;
    };

    // Prefetch touches, one 128-byte line per lane: the workgroup's quarter of its A panel's rows (the 4 tiles
    // beside it along n read the same panel) and its eighth of its B panel's rows (8 tiles along m).  Contiguous
    // along k: lanes 0 .. 2 IM - 1 take A rows 8 IM (tile_n % 4) + 2 IM w + lane, the next JN lanes take B rows
    // 4 JN (tile_m % 8) + JN w + (lane - 2 IM).  Contiguous along m / n (a K-tile is 64 k-rows of IM / 2 lines, JN / 2
    // for B): the same number of lanes take A k-rows 16 (tile_n % 4) + 4 w + lane / (IM / 2), line lane % (IM / 2),
    // and B k-rows 8 (tile_m % 8) + 2 w + u / (JN / 2), line u % (JN / 2), u = lane - 2 IM.  The remaining lanes repeat
    // lane 0 and coalesce with it.
    const char *touch_ptr;
    int64_t touch_step;
    {
        constexpr int kTouchA = 2 * IM, kTouchB = JN;
        const int tl = lane < kTouchA + kTouchB ? lane : 0, u = tl - kTouchA;
        if (tl < kTouchA) {
            touch_ptr = AMC ? reinterpret_cast<const char *>(A + (int64_t)((tile_n & 3) * 16 + wave * 4 + tl / (IM / 2)) * g.lda + m0 + (tl % (IM / 2)) * 64)
                            : reinterpret_cast<const char *>(A + (int64_t)(m0 + (tile_n & 3) * (8 * IM) + wave * (2 * IM) + tl) * g.lda);
            touch_step = AMC ? kstep_a : kBK * 2;
        } else {
            touch_ptr = BMC ? reinterpret_cast<const char *>(B + (int64_t)((tile_m & 7) * 8 + wave * 2 + u / (JN / 2)) * g.ldb + n0 + (u % (JN / 2)) * 64)
                            : reinterpret_cast<const char *>(B + (int64_t)(n0 + (tile_m & 7) * (4 * JN) + wave * JN + u) * g.ldb);
            touch_step = BMC ? kstep_b : kBK * 2;
        }
    }
    const uint32_t touch_lds = lds0 + 2 * kStageBytes + wave * 256;
    auto touch_m0 = [&]() {
        const uint32_t w = touch_lds;
        asm volatile("s_mov_b32 m0, %0" ::"s"(w) : "m0");
    };
    auto touch_go = [&](int t) {
        const int tc = t < nk ? t : nk - 1;
        const char *p = touch_ptr + (int64_t)tc * touch_step;
        asm volatile("global_load_lds_dword %0, off" ::"v"(p) : "memory");
    };

    // Fragment addresses.  Contiguous along k: row l16 of the block, chunk 4 kk + lq; blocks are 2 KB apart.
    // Contiguous along m / n: as the source of a transposing read the lane points at k-row
    // k = 32 kk + 8 lq + 4 h + l16 / 4 (h = 0, 1: the two reads), rows 16 b + 4 (l16 % 4) .. + 3 of the wavefront's
    // part.  K-row k of sub-tile u lies in the KB that wavefront k / 16 filled with its load 2 u + (k / 8) % 2, 128
    // bytes per k-row, chunks swizzled by kswz(k) (which 4 h and 32 kk leave alone); block g of the tile's 2 IM is
    // chunks 2 (g % 4), + 1 of sub-tile g / 4.  One address per lane and block; k-step and half add 2 IM KB and 512.
    int ra_off[2], rb_off[2], ra_blk[AMC ? IM : 1], rb_blk[BMC ? JN : 1];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int pos = (4 * kk + lq) ^ ((l16 >> 1) & 7);
        ra_off[kk] = (wm0 + l16) * 128 + pos * 16;
        rb_off[kk] = kTileA + (wn0 + l16) * 128 + pos * 16;
    }
    {
        const int krow = 8 * lq + (l16 >> 2), half = (l16 >> 1) & 1;
        const int in_kb = (krow & 7) * 128 + ((half ^ kswz(krow)) * 16) + (l16 & 1) * 8;
        if constexpr (AMC) {
#pragma unroll
            for (int b = 0; b < IM; ++b) {
                const int gb = wm0 / 16 + b;
                ra_blk[b] = ((krow >> 4) * IM + 2 * (gb >> 2) + ((krow >> 3) & 1)) * 1024 + (in_kb ^ ((gb & 3) << 5));
            }
        }
        if constexpr (BMC) {
#pragma unroll
            for (int b = 0; b < JN; ++b) {
                const int gb = wn0 / 16 + b;
                rb_blk[b] = kTileA + ((krow >> 4) * JN + 2 * (gb >> 2) + ((krow >> 3) & 1)) * 1024 + (in_kb ^ ((gb & 3) << 5));
            }
        }
    }
    bf16x8 Fa[2][IM], Fb[2][JN];        // [k-step][block row / column]
    auto tr_read = [&](const char *p) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FSR_AS3 s16x4 *)(FSR_AS3 char *)p);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FSR_AS3 s16x4 *)(FSR_AS3 char *)(p + 512));
        return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // fragment r of k-step kk of the K-tile in `stage` (r < IM: a_r, else b_(r - IM)) into the registers of k-step kd
    auto lread = [&](int stage, int kk, int kd, int r) {
        const char *s = smem + stage * kStageBytes;
        if (r < IM) {
            if constexpr (AMC) Fa[kd][r] = tr_read(s + ra_blk[r] + kk * (2048 * IM));
            else Fa[kd][r] = *reinterpret_cast<const bf16x8 *>(s + ra_off[kk] + r * 2048);
        } else {
            const int j = r - IM;
            if constexpr (BMC) Fb[kd][j] = tr_read(s + rb_blk[j] + kk * (2048 * JN));
            else Fb[kd][j] = *reinterpret_cast<const bf16x8 *>(s + rb_off[kk] + j * 2048);
        }
    };

    f32x4 acc[IM][JN];

    constexpr int kTouchSlot = kLoadEvery * kLate + 1;      // behind the late loads, so the touch is the youngest load at the barrier
    static_assert(kLoadEvery * (kEarly - 1) + 2 < kMfmas && kTouchSlot + 2 < kMfmas, "slots of one half");
    using Chain = ChainPlan<IM, JN, kLate, kEarly, kLoadEvery, kTouchSlot>;

    // K-tile t in stage P: its walk is P's (0 row by row, 1 column by column); half 0 is slots 0 .. kMfmas - 1
    auto k_tile = [&](auto parity, int t) {
        constexpr int P = decltype(parity)::value;
        constexpr int X = P, Y = 1 - P;
        static_for<2>([&](auto hc) {
            constexpr int h = decltype(hc)::value;
            static_for<kMfmas>([&](auto mc) {
                constexpr int m = decltype(mc)::value;
                constexpr int slot = h * kMfmas + m, blk = slot / 2, kk = slot % 2;
                constexpr int i = Chain::blk_i(P, blk), j = Chain::blk_j(P, blk);
                constexpr int c = m / kLoadEvery;               // load of this group of slots
                constexpr bool has_load = h == 1 ? c < kEarly : c < kLate;
                if constexpr (m % kLoadEvery == 1 && has_load) {
                    if constexpr (h == 1) load_m0(Int<X>{}, Int<c>{});
                    else load_m0(Int<Y>{}, Int<kEarly + c>{});
                }
                if constexpr (h == 0 && m == kTouchSlot) touch_m0();
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(Fa[kk][i]), "v"(Fb[kk][j]));
                // half 0: the last fragments of this K-tile (from X, into registers the K-tile before has freed);
                // half 1: the first fragments of the next K-tile (from Y, complete since the barrier)
                constexpr int f = h == 0 ? Chain::kPlan[1 - P].frag[kMfmas + m] : Chain::kPlan[P].frag[m];
                if constexpr (f >= 0) lread(h == 0 ? X : Y, Chain::kk_of(f), Chain::kk_of(f), f % (IM + JN));
                if constexpr (m % kLoadEvery == 2 && has_load) {
                    if constexpr (h == 1) load_go(Int<c>{});
                    else load_go(Int<kEarly + c>{});
                }
                if constexpr (h == 0 && m == kTouchSlot + 1) touch_go(t + kTouchAhead);
                if constexpr (h == 0 && m == kTouchSlot + 2) advance(t + 2);
                __builtin_amdgcn_sched_barrier(0);
            });
            if constexpr (h == 0) {
                // All loads but the youngest (the touch) have landed: K-tile t+1 is complete in Y.  Every
                // wavefront also has all fragments of X in registers, so after the barrier Y may be read and X
                // overwritten.  The LDS counter is drained through the builtin so that the compiler, which
                // places the waits in front of the MFMAs that use a fragment, knows it.
                asm volatile("s_waitcnt vmcnt(1)" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0xC07F);             // lgkmcnt(0)
                __builtin_amdgcn_s_barrier();
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // Prologue: K-tile 0 into stage 0 and touches for the K-tiles the loop's own touches come too late for;
    // only K-tile 0 is waited for (the touches are the youngest kTouchAhead - 1 loads).
    static_for<kLoads>([&](auto ic) {
        load_m0(Int<0>{}, ic);
        asm volatile("s_nop 0");
        load_go(ic);
    });
    touch_m0();
    asm volatile("s_nop 0");
#pragma unroll
    for (int p = 1; p < kTouchAhead; ++p) touch_go(p);
    advance(1);
    // the accumulators are cleared while K-tile 0 is on its way
#pragma unroll
    for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int j = 0; j < JN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int j = 0; j < JN; ++j) asm volatile("" : "+a"(acc[i][j]));      // pins the clears here
    __builtin_amdgcn_sched_barrier(0);
    static_assert(kTouchAhead == 3 || kTouchAhead == 4, "the wait below skips the kTouchAhead - 1 touches");
    if constexpr (kTouchAhead == 3) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // then the early loads of K-tile 1 into stage 1 and all fragments of K-tile 0 (its first half reads some again)
    static_for<kEarly>([&](auto ic) {
        load_m0(Int<1>{}, ic);
        asm volatile("s_nop 0");
        load_go(ic);
    });
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int r = 0; r < kReads; ++r) lread(0, kk, kk, r);
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_sched_barrier(0);

    int t = 0;
    for (; t + 1 < nk; t += 2) {
        k_tile(Int<0>{}, t);
        k_tile(Int<1>{}, t + 1);
    }
    if (t < nk) k_tile(Int<0>{}, t);

    // The rest of K: one more K-tile into stage 0, outside the pipeline.  The lane that fills position p of a row
    // fetches the piece that belongs there if it lies inside K, else the zero piece.
    const int k_rest = g.K - nk * kBK;
    if (k_rest > 0) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();       // every load has landed and every wavefront is done with both stages
        __builtin_amdgcn_sched_barrier(0);
        // (the lane id is taken afresh from the hardware: nothing of this step is to be worked out, and kept in registers, ahead of the loop)
        int ln = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        asm volatile("" : "+v"(ln));
        auto rest_src = [&](auto mcc, const uint16_t *P, int64_t ld, int origin, int rows_per_wave, int q) -> const uint16_t * {
            if constexpr (decltype(mcc)::value) {
                const int kr = wave * 16 + (q & 1) * 8 + (ln >> 3);       // k-row of the K-tile, in sub-tile q / 2
                return kr < k_rest ? P + (int64_t)(nk * kBK + kr) * ld + origin + 64 * (q >> 1) + 8 * ((ln & 7) ^ kswz(kr)) : kZeroPiece;
            } else {
                const int row = ln >> 3, chunk = (ln & 7) ^ (((row >> 1) & 3) | ((q & 1) << 2));
                return 8 * chunk < k_rest ? P + (int64_t)(origin + wave * rows_per_wave + q * 8 + row) * ld + nk * kBK + 8 * chunk : kZeroPiece;
            }
        };
#pragma unroll
        for (int idx = 0; idx < kLoads; ++idx) {
            const bool is_a = idx < kLoadsA;
            const int q = is_a ? idx : idx - kLoadsA;
            char *dst = smem + (is_a ? wave * (kLoadsA * 1024) : kTileA + wave * (kLoadsB * 1024)) + q * 1024;
            const uint16_t *src = is_a ? rest_src(std::integral_constant<bool, AMC>{}, A, g.lda, m0, 8 * IM, q)
                                       : rest_src(std::integral_constant<bool, BMC>{}, B, g.ldb, n0, 8 * JN, q);
            __builtin_amdgcn_global_load_lds((const FSR_AS1 void *)src, (FSR_AS3 void *)dst, 16, 0, 0);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            if (32 * kk < k_rest) {
#pragma unroll
                for (int r = 0; r < kReads; ++r) lread(0, kk, 0, r);
                __builtin_amdgcn_s_waitcnt(0xC07F);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int m = 0; m < kMfmas; ++m)
                    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[m / JN][m % JN]) : "v"(Fa[0][m / JN]), "v"(Fb[0][m % JN]));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    // no load may still be writing LDS when the wavefront ends, and the last MFMAs must have retired
    // before the accumulators are read (the compiler does not know what wrote them)
    asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");

    // Register r of a 16x16 block holds row 4 (lane / 16) + r, column lane % 16.  The lane id is taken
    // afresh from the hardware so that no store address is kept in a register across the loop; blocks are fenced so that the
    // accumulators are copied out a block at a time.
    float *__restrict__ C = g.C;
    int lane_e = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));      // the lane's number within its wavefront
    asm volatile("" : "+v"(lane_e));
    const int l16e = lane_e & 15, lqe = lane_e >> 4;
#pragma unroll
    for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int j = 0; j < JN; ++j) {
            const int col = n0 + wn0 + j * 16 + l16e;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = m0 + wm0 + i * 16 + lqe * 4 + r;
                C[(int64_t)row * g.ldc + col] = acc[i][j][r];
            }
            __builtin_amdgcn_sched_barrier(0);
        }
}

}  // namespace

// in the order of the candidate numbers: 256 x 256 was there first
constexpr int kShapeM[kBf16MainShapes] = {256, 192, 128, 256, 192, 256, 128}, kShapeN[kBf16MainShapes] = {256, 256, 256, 192, 192, 128, 128};

int bf16_main_tile_m(int shape) { return kShapeM[shape]; }
int bf16_main_tile_n(int shape) { return kShapeN[shape]; }

// <blocks of 16 rows per wavefront, blocks of 16 columns, A layout, B layout> with 0 = contiguous along k, 1 = along
// m / n; as a profiler trace prints the kernel
const char *bf16_main_kernel_name(int shape, int a_lay, int b_lay)
{
    struct Names {
        char text[kBf16MainShapes][2][2][40];
        Names()
        {
            for (int sh = 0; sh < kBf16MainShapes; ++sh)
                for (int a = 0; a < 2; ++a)
                    for (int b = 0; b < 2; ++b)
                        snprintf(text[sh][a][b], sizeof text[sh][a][b], "gemm_bf16_main_kernel<%d, %d, %d, %d>", kShapeM[sh] / 32, kShapeN[sh] / 32, a, b);
        }
    };
    static const Names names;
    return names.text[shape][a_lay][b_lay];
}

// Whole unchecked tiles of 16-byte pieces: a matrix at least one tile high and wide (a ragged last tile is shifted
// back into it), at least one whole K-tile of 64 and K a multiple of 8 (the rest of K is whole pieces), 16-byte aligned
// bases and rows, leading dimensions below 2^25 (32-bit lane offsets); an operand that is contiguous along m (n) needs
// M (N) a multiple of 8, so that a shifted tile still starts on a piece.
bool bf16_main_fits(int shape, int a_lay, int b_lay, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb)
{
    if (shape < 0 || shape >= kBf16MainShapes) return false;
    const int bm = kShapeM[shape], bn = kShapeN[shape];
    const bool aligned = ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 15u) == 0 && lda % 8 == 0 && ldb % 8 == 0;
    return aligned && lda < (1 << 25) && ldb < (1 << 25) && M >= bm && N >= bn && K >= kBK && K % 8 == 0 &&
           (a_lay == kKContig || M % 8 == 0) && (b_lay == kKContig || N % 8 == 0) &&
           ((M + bm - 1) / bm) * ((N + bn - 1) / bn) < ((int64_t)1 << 31);
}

namespace {

template <int IM, int JN, int ALAY, int BLAY>
hipError_t launch_main(const GemmArgs &a, hipStream_t s)
{
    constexpr int kLdsBytes = 2 * (32 * IM + 32 * JN) * kBK * 2 + kScratchBytes;
    auto kern = gemm_bf16_main_kernel<IM, JN, ALAY, BLAY>;
    static std::atomic<uint64_t> configured{0};
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), kLdsBytes, configured);
    if (e != hipSuccess) return e;
    const int tiles_m = (a.M + 32 * IM - 1) / (32 * IM), tiles_n = (a.N + 32 * JN - 1) / (32 * JN);
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n * a.k_slices)), dim3(kThreads), kLdsBytes, s, a, tiles_m, tiles_n);
    return hipGetLastError();
}

template <int IM, int JN>
hipError_t launch_shape(int a_lay, int b_lay, const GemmArgs &a, hipStream_t s)
{
    if (a_lay == kKContig && b_lay == kKContig) return launch_main<IM, JN, kKContig, kKContig>(a, s);
    if (a_lay == kMnContig && b_lay == kKContig) return launch_main<IM, JN, kMnContig, kKContig>(a, s);
    if (a_lay == kKContig && b_lay == kMnContig) return launch_main<IM, JN, kKContig, kMnContig>(a, s);
    if (a_lay == kMnContig && b_lay == kMnContig) return launch_main<IM, JN, kMnContig, kMnContig>(a, s);
    return hipErrorInvalidValue;
}

}  // namespace

// K may be cut into `slices` whole numbers of K-tiles if the last slice still has a whole K-tile
bool bf16_main_slices_fit(int64_t K, int slices)
{
    return slices >= 1 && K < ((int64_t)1 << 31) && (int64_t)(slices - 1) * bf16_main_slice_length((int)K, slices) + kBK <= K;
}

// requires bf16_main_fits(...) and bf16_main_slices_fit(a.K, a.k_slices); with slices, a.C is the workspace and a.ldc = a.N
hipError_t launch_bf16_main(int shape, int a_lay, int b_lay, const GemmArgs &a, hipStream_t s)
{
    if (!bf16_main_fits(shape, a_lay, b_lay, a.M, a.N, a.K, a.A, a.lda, a.B, a.ldb) || !bf16_main_slices_fit(a.K, a.k_slices)) return hipErrorInvalidValue;
    if (((a.M + kShapeM[shape] - 1) / kShapeM[shape]) * (int64_t)((a.N + kShapeN[shape] - 1) / kShapeN[shape]) * a.k_slices >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    switch (shape) {
    case 0: return launch_shape<8, 8>(a_lay, b_lay, a, s);
    case 1: return launch_shape<6, 8>(a_lay, b_lay, a, s);
    case 2: return launch_shape<4, 8>(a_lay, b_lay, a, s);
    case 3: return launch_shape<8, 6>(a_lay, b_lay, a, s);
    case 4: return launch_shape<6, 6>(a_lay, b_lay, a, s);
    case 5: return launch_shape<8, 4>(a_lay, b_lay, a, s);
    default: return launch_shape<4, 4>(a_lay, b_lay, a, s);
    }
}

}  // namespace fsrgemm
