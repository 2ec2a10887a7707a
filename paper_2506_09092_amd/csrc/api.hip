// C ABI of the library (declared in include/fsrgemm.h): argument checks,
// choice of tile configuration and load mode, launch on the caller's stream.
#include "../../include/fsrgemm.h"

#include <stdio.h>
#include <string.h>

#include "launchers.hpp"

using namespace fsrgemm;

namespace {

struct Plan {
    int cfg;        // tile configuration (F32Config / Bf16Config)
    int mode;       // load mode, follows from the tile, the shape and the alignment
    int slices;     // K slices of a call that brings a workspace; 1 = one piece
    // Two bands (direct-to-LDS shapes only): rows (band_dim 1) or columns (2) [0, band_at) of C run as configuration
    // cfg, the rest as cfg2, one launch each on the caller's stream; 0 = one launch
    int band_dim = 0;
    int64_t band_at = 0;
    int cfg2 = 0;
};

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks shared by all entry points.  lda_min / ldb_min are the extents of the operands' contiguous index (K or M
// for A, N or K for B, by storage order).  Returns FSRGEMM_OK when the problem is well formed.
int check_args(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, int64_t lda_min, const void *B,
               int64_t ldb, int64_t ldb_min, const void *C, int64_t ldc)
{
    const int64_t lim = (int64_t)1 << 31;
    if (M < 0 || N < 0 || K < 0 || M >= lim || N >= lim || K >= lim) return FSRGEMM_ERR_INVALID_ARG;
    if (lda < lda_min || ldb < ldb_min || ldc < N) return FSRGEMM_ERR_INVALID_ARG;
    if (M > 0 && N > 0 && C == nullptr) return FSRGEMM_ERR_INVALID_ARG;
    if (M > 0 && N > 0 && K > 0 && (A == nullptr || B == nullptr)) return FSRGEMM_ERR_INVALID_ARG;
    return FSRGEMM_OK;
}

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Configurations that the selection loop found faster than the rules below, by exact problem: the incumbent
// (k_best) of the paper's Algorithm 1 with tile configurations and K slices as the candidates.  A row with
// ws == 0 serves calls without a workspace (its slices are 1), a row with ws == 1 calls that bring one.
struct Tuned {
    int kind;       // 0 = fp32, 1 = bf16
    int transA, transB;
    int M, N, K;
    int ws;
    int tile, slices;
};
constexpr Tuned kTuned[] = {
#include "tuned_table.inc"
    {-1, 0, 0, 0, 0, 0, 0, 0, 0}};

const Tuned *find_tuned(int kind, int transA, int transB, int64_t M, int64_t N, int64_t K, bool ws)
{
    for (const Tuned &t : kTuned)
        if (t.kind == kind && (ws || t.slices == 1) && (ws || kind != 0 || t.tile != kF32_Skinny) &&      // never a row that needs a workspace for a call without one
             t.M == M && t.N == N && t.K == K && t.transA == (transA != 0) && t.transB == (transB != 0) &&
            t.ws == (int)ws)
            return &t;
    return nullptr;
}

constexpr int kF32TileM[kF32ConfigCount] = {256, 128, 64}, kF32TileN[kF32ConfigCount] = {128, 128, 64};
constexpr int kBf16Tile[kBf16ConfigCount] = {256, 256, 128, 64};
constexpr int kMaxSlices = 64;
constexpr int64_t kMaxWorkspace = (int64_t)16 << 20;

// Split-K rule: problems with few 64 x 64 output tiles and a long K are cut into K slices so that about 1024
// workgroups stream the operands.  A slice keeps at least 256 k when the tiles alone leave half the compute
// units idle, 1024 k when they would fill them once or twice; at most 64 slices, partial products within
// 16 MiB.  Depends on the shape only, so the order of summation, and with it the result, is the same on every
// call.  k_tile = 16 for fp32, 64 for bf16.  1 = do not split.
int splitk_slices(int64_t M, int64_t N, int64_t K, int k_tile)
{
    const int64_t tiles = ceil_div(M, 64) * ceil_div(N, 64), nk = ceil_div(K, k_tile);
    if (M == 0 || N == 0 || tiles > 512) return 1;
    int64_t s = 1024 / tiles;
    const int64_t longest = nk / ((tiles <= 128 ? 256 : 1024) / k_tile);
    if (s > longest) s = longest;
    if (s > kMaxSlices) s = kMaxSlices;
    const int64_t cap = kMaxWorkspace / (M * N * 4);
    if (s > cap) s = cap;
    return s < 2 ? 1 : (int)s;
}

// Load mode of an fp32 tile configuration for this problem.  Unchecked loads and stores need whole K-tiles and a
// matrix at least one tile wide and high (a ragged last tile is shifted back into the matrix).  Grids beyond
// 2^31 - 1 workgroups are rejected.
int mode_f32(int cfg, int slices, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
             int *mode)
{
    if (cfg == kF32_Skinny || cfg >= kF32_Main) {      // whether they fit the problem is their own check
        *mode = 0;
        return FSRGEMM_OK;
    }
    if (cfg == kF32_Vector) {           // the vector kernels look at alignment themselves
        *mode = 0;
        return ceil_div(M > N ? M : N, 4) * slices >= ((int64_t)1 << 31) ? FSRGEMM_ERR_INVALID_ARG : FSRGEMM_OK;
    }
    const int bm = kF32TileM[cfg], bn = kF32TileN[cfg];
    if (ceil_div(M, bm) * ceil_div(N, bn) * slices >= ((int64_t)1 << 31)) return FSRGEMM_ERR_INVALID_ARG;
    const bool vec = aligned16(A) && aligned16(B) && lda % 4 == 0 && ldb % 4 == 0;
    const bool near = lda < kF32MaxLdUnchecked && ldb < kF32MaxLdUnchecked;      // 32-bit lane offsets of the unchecked loads
    *mode = !vec ? kScalar : (M >= bm && N >= bn && K % 16 == 0 && K > 0 && near) ? kFast : kVecPred;
    return FSRGEMM_OK;
}

// Tile rule for fp32: the configuration with the least modelled time.  A compute unit works through its share
// of the output tiles at a rate that depends on the tile only, so a launch takes ceil(tiles / 256) tile times
// (256 compute units; a last round with few tiles costs a whole one), and never less than the time of one
// workgroup running alone.  Times per tile and k step, in units of 0.1 ns, measured on square problems with
// each configuration forced: 256 x 128: 1137, 128 x 128: 569, 64 x 64: 169 with several workgroups per compute
// unit, 221 alone.  K cancels.  Equal costs go to the larger tile.  The shapes of the direct-to-LDS kernel (main_fits:
// bit s set if shape s can take the problem) enter with their own tile times and win where their tiles fill whole
// rounds; its tiles with a side of 64 (148 / 290 / 300 for 64 x 64, 128 x 64, 64 x 128: within 7 % of the 256 x 256
// tile's time per flop, several workgroups sharing a compute unit) take the problems of 1024 ... 2560 rows that the
// general 64 x 64 tile ran before.
constexpr int64_t kMainTileTime[kF32MainShapes] = {2230, 1710, 1120, 1120, 838, 566, 1715, 1286, 845, 148, 290, 300};   // in the order of the shapes
int tile_rule_f32(int64_t M, int64_t N, unsigned main_fits, int64_t *cost_out = nullptr)
{
    constexpr int64_t kTileTime[kF32ConfigCount] = {1137, 569, 169}, kAlone[kF32ConfigCount] = {1137, 569, 221};
    int best = 0;
    int64_t best_cost = 0;
    for (int c = 0; c < kF32ConfigCount; ++c) {
        const int64_t rounds = ceil_div(ceil_div(M, kF32TileM[c]) * ceil_div(N, kF32TileN[c]), 256);
        int64_t cost = rounds * kTileTime[c];
        if (cost < kAlone[c]) cost = kAlone[c];
        if (c == 0 || cost < best_cost) best = c, best_cost = cost;
    }
    for (int sh = 0; sh < kF32MainShapes; ++sh) {
        if (!(main_fits >> sh & 1)) continue;
        const int64_t cost = ceil_div(ceil_div(M, f32_main_tile_m(sh)) * ceil_div(N, f32_main_tile_n(sh)), 256) * kMainTileTime[sh];
        if (cost < best_cost) best = kF32_Main + sh, best_cost = cost;
    }
    if (cost_out) *cost_out = best_cost;
    return best;
}

// K slices on the direct-to-LDS shapes, for calls that bring a workspace: the shape and slice count with the least modelled
// time.  With w = ceil(tiles x slices / 256) workgroups to a compute unit one after (or beside) the other, each over a
// slice of L k, a launch takes w L t: t the shape's tile time, or, for the 64-wide shapes with a unit to themselves, the
// time of a workgroup running alone (161 / 301 / 324); plus 1 us per workgroup in a unit's queue for what surrounds its K
// loop, and for slices the second launch (4 us) and its traffic (slices + 1 results at 3 TB/s); a slice keeps 256 k or more.  Measured against the
// plans this replaced (64 x 64 and 128 x 128 tiles of the general kernel in up to 64 slices): 256^2 x 16384 39 -> 26 us,
// 512^2 x 4096 28 -> 23, 768^2 x 2048 41 -> 28, 1024^2 x 2048 42 -> 34 (unsplit), 128 x 2048 x 4096 29 -> 23.
// A split is taken for a modelled gain of 5 % over the best unsplit shape.  Units of 0.1 ns.
struct MainSplit {
    int shape = -1, slices = 1;
    double cost = 0;        // (a double: tiles x K x tile time leaves 64 bits for extents near their limits)
};
MainSplit best_main_split(int64_t M, int64_t N, int64_t K, unsigned main_fits)
{
    constexpr int64_t kAlone[kF32MainShapes] = {2230, 1710, 1120, 1120, 838, 566, 1715, 1286, 845, 161, 301, 324};
    MainSplit best, unsplit;
    for (int sh = 0; sh < kF32MainShapes; ++sh) {
        if (!(main_fits >> sh & 1)) continue;
        const int64_t tiles = ceil_div(M, f32_main_tile_m(sh)) * ceil_div(N, f32_main_tile_n(sh));
        for (int sl = 1; sl <= kMaxSlices; ++sl) {
            if (sl > 1 && (int64_t)sl * M * N * 4 > kMaxWorkspace) break;
            if (!f32_main_slices_fit(K, sl)) continue;       // the last slice would be left without a whole K-tile
            const int64_t w = ceil_div(tiles * sl, 256), len = ceil_div(ceil_div(K, 32), sl) * 32;
            double cost = (double)w * (double)len * (double)(w == 1 ? kAlone[sh] : kMainTileTime[sh]) + (double)w * 10000.0;
            if (sl > 1 && len < 256) continue;                // a slice keeps at least eight K-tiles
            if (sl > 1) cost += 40000.0 + (double)(sl + 1) * (double)M * (double)N * 4.0 / 300.0;
            if (sl == 1 && (unsplit.shape < 0 || cost < unsplit.cost)) unsplit.shape = sh, unsplit.cost = cost;
            if (best.shape < 0 || cost < best.cost) best.shape = sh, best.slices = sl, best.cost = cost;
        }
    }
    return best.slices > 1 && best.cost > unsplit.cost * 0.95 ? unsplit : best;
}

// Two bands.  Where no tile shape fills whole rounds of the compute units, two launches often do: C is cut once, along
// its rows or its columns, and each band takes the shape that suits its own tile count (fp32 5120^2: 729 tiles of
// 192 x 192 are 2.85 rounds; rows 0 .. 1023 as 1280 tiles of 64 x 64 and the rest as 1280 tiles of 128 x 128 are five whole
// rounds each and take 9 % less time).  The bands are independent products on shifted pointers, so nothing changes in a kernel and every
// entry of C is still computed by one workgroup in the same order of summation.  cost(shape, m, n) is the modelled
// time of an m x n band in that shape, negative where the shape cannot take it; cuts are multiples of 64 (every tile
// side is one, and a cut then keeps the operands' alignment), at most 256 per direction.
struct Bands {
    int dim = 0;
    int64_t at = 0;
    int sh1 = -1, sh2 = -1;
    int64_t cost = 0;
};
// The search is a few thousand cost evaluations (tens of microseconds), and callers repeat their problems: the last
// results are kept per thread, keyed by everything the search depends on (precision and storage orders, extents, which
// shapes fit the problem).
struct BandsKey {
    int kind, lays;
    int64_t M, N, K;
    unsigned fits;
    bool operator==(const BandsKey &o) const { return kind == o.kind && lays == o.lays && M == o.M && N == o.N && K == o.K && fits == o.fits; }
};
template <class Cost>
Bands best_bands(const BandsKey &key, int shapes, Cost cost, int64_t launch_gap)
{
    constexpr int kSlots = 16;
    struct Slot {
        bool used = false;
        BandsKey key;
        Bands bands;
    };
    static thread_local Slot cache[kSlots];
    Slot &slot = cache[(uint64_t)(key.M * 31 + key.N * 17 + key.K * 7 + key.kind * 3 + key.lays) % kSlots];
    if (slot.used && slot.key == key) return slot.bands;
    const int64_t M = key.M, N = key.N;
    Bands best;
    for (int dim = 1; dim <= 2; ++dim) {
        const int64_t ext = dim == 1 ? M : N;
        const int64_t step = 64 * ceil_div(ext, 64 * 256);
        for (int64_t at = 64; at + 64 <= ext; at += step) {
            int s1 = -1, s2 = -1;
            int64_t c1 = 0, c2 = 0;
            for (int sh = 0; sh < shapes; ++sh) {
                const int64_t a = dim == 1 ? cost(sh, at, N) : cost(sh, M, at), b = dim == 1 ? cost(sh, ext - at, N) : cost(sh, M, ext - at);
                if (a >= 0 && (s1 < 0 || a < c1)) s1 = sh, c1 = a;
                if (b >= 0 && (s2 < 0 || b < c2)) s2 = sh, c2 = b;
            }
            if (s1 < 0 || s2 < 0 || s1 == s2) continue;      // two bands of one shape are the one launch cut in two
            const int64_t c = c1 + c2 + launch_gap;
            if (best.dim == 0 || c < best.cost) best.dim = dim, best.at = at, best.sh1 = s1, best.sh2 = s2, best.cost = c;
        }
    }
    slot.used = true, slot.key = key, slot.bands = best;
    return best;
}

// Operands and result of the band that starts at row (dim 1) or column (dim 2) `at` of C.  The planners call this with
// whatever they were given for A and B (possibly NULL: only the alignment is looked at), hence addresses as integers.
template <class T>
void shift_to_band(int dim, int64_t at, int a_lay, int b_lay, const T *&A, int64_t lda, const T *&B, int64_t ldb, float *&C, int64_t ldc)
{
    const int64_t off_a = dim == 1 ? (a_lay == kKContig ? at * lda : at) : 0, off_b = dim == 2 ? (b_lay == kKContig ? at * ldb : at) : 0;
    const int64_t off_c = dim == 1 ? at * ldc : at;
    A = reinterpret_cast<const T *>(reinterpret_cast<uintptr_t>(A) + (uintptr_t)off_a * sizeof(T));
    B = reinterpret_cast<const T *>(reinterpret_cast<uintptr_t>(B) + (uintptr_t)off_b * sizeof(T));
    C = reinterpret_cast<float *>(reinterpret_cast<uintptr_t>(C) + (uintptr_t)off_c * sizeof(float));
}

// How a product with M == 1 or N == 1 (or with a few rows or columns on the smaller side: kMaxFewVectorsF32, kMaxFewVectors, kMaxMfmaVectors) maps onto
// the vector kernels: which operand is the matrix, how it is walked, and the strides of the vectors on either side.
// ARGS: VecArgs (fp32) or VecArgs16 (bf16); T the element type.
template <class ARGS, class T>
struct VecMapT {
    int pattern;
    ARGS a;
};
template <class ARGS, class T>
VecMapT<ARGS, T> vector_map_t(int transA, int transB, int64_t M, int64_t N, int64_t K, const T *A, int64_t lda, const T *B,
                              int64_t ldb, float *C, int64_t ldc)
{
    VecMapT<ARGS, T> v;
    v.a.K = (int)K;
    v.a.k_slices = 1;
    v.a.slice_stride = 0;
    v.a.xvec = false;
    if (N <= M) {       // a matrix times columns: y = C's columns, x = B's
        v.pattern = transA ? kVecCols : kVecRows;
        v.a.mat = A, v.a.ld = lda, v.a.len = (int)M;
        v.a.x = B, v.a.incx = transB ? 1 : ldb, v.a.ldx = transB ? ldb : 1;
        v.a.y = C, v.a.incy = ldc, v.a.ldy = 1;
        v.a.nvec = (int)N;
    } else {            // rows times a matrix: y = C's rows, x = A's
        v.pattern = transB ? kVecRows : kVecCols;
        v.a.mat = B, v.a.ld = ldb, v.a.len = (int)N;
        v.a.x = A, v.a.incx = transA ? lda : 1, v.a.ldx = transA ? 1 : lda;
        v.a.y = C, v.a.incy = 1, v.a.ldy = ldc;
        v.a.nvec = (int)M;
    }
    return v;
}
using VecMap = VecMapT<VecArgs, float>;
VecMap vector_map(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                  int64_t ldb, float *C, int64_t ldc)
{
    return vector_map_t<VecArgs, float>(transA, transB, M, N, K, A, lda, B, ldb, C, ldc);
}
using VecMap16 = VecMapT<VecArgs16, uint16_t>;
VecMap16 vector_map16(int transA, int transB, int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda,
                      const uint16_t *B, int64_t ldb, float *C, int64_t ldc)
{
    return vector_map_t<VecArgs16, uint16_t>(transA, transB, M, N, K, A, lda, B, ldb, C, ldc);
}

// Workgroups of the vector kernels for an output of `len` elements, and the K slices of a call with a
// workspace.  A split costs a second launch, so K is cut only to reach enough workgroups to keep the memory
// system busy, and never finer than 2048 (1024 for the column pattern): 256 workgroups, or 1024 for the bf16 column pattern
// on a matrix of 128 MiB and more, whose workgroups each keep 32 KB in flight, 512 for that pattern with several vectors
// (the selection loop: 4 x 8192 x 8192 and 8192 x 4 x 8192 3 - 4 % faster in 4 slices than in 2) (measured: fp32 1 x 4096 x 4096 gains 15 % from
// two slices, 1 x 8192 x 8192 loses 15 % to two, 1 x 1024 x 1024 loses 40 % to any split; bf16 1 x 16384 x 16384 with a row-major
// B gains 35 % from four).
int64_t vector_groups(int pattern, int64_t len, int cols_per_group, int rows_per_group = 4) { return pattern == kVecRows ? ceil_div(len, rows_per_group) : ceil_div(len, cols_per_group); }
int vector_slices(int pattern, int64_t len, int64_t K, int cols_per_group = 32, int rows_per_group = 4)
{
    const int64_t matrix_bytes = len * K * (cols_per_group == 32 ? 4 : 2);
    const int64_t target = pattern == kVecCols && cols_per_group == 64 ? (rows_per_group != 4 ? 512 : matrix_bytes >= ((int64_t)128 << 20) ? 1024 : 256) : 256;
    int64_t s = target / vector_groups(pattern, len, cols_per_group, rows_per_group);
    const int64_t shortest = pattern == kVecCols ? 1024 : 2048;
    if (s > K / shortest) s = K / shortest;
    if (s > kMaxSlices) s = kMaxSlices;
    return s < 2 ? 1 : (int)s;
}

// (K beyond 2^30 stays with the tile kernels: the vector kernels count k in 32-bit steps of up to 1024)
bool vector_shape(int64_t M, int64_t N, int64_t K) { return (M == 1 || N == 1) && M > 0 && N > 0 && K > 0 && K <= ((int64_t)1 << 30); }
// fp32 also with 2 .. kMaxFewVectorsF32 rows or columns on the smaller side, where the other operand (the matrix that is
// streamed) consists of aligned 16-byte pieces
bool vector_call_f32(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb)
{
    if (vector_shape(M, N, K)) return true;
    if (M < 1 || N < 1 || K < 1 || K > ((int64_t)1 << 30) || (M > kMaxFewVectorsF32 && N > kMaxFewVectorsF32)) return false;
    const VecMap v = vector_map(transA, transB, M, N, K, A, lda, B, ldb, nullptr, 1);
    return gemv_takes_few(v.pattern, v.a);
}

bool vector_call_bf16(int transA, int transB, int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb)
{
    if (vector_shape(M, N, K)) return true;
    if (M < 1 || N < 1 || K < 1 || K > ((int64_t)1 << 30) || (M > kMaxMfmaVectors && N > kMaxMfmaVectors)) return false;
    const VecMap16 v = vector_map16(transA, transB, M, N, K, A, lda, B, ldb, nullptr, 1);
    return gemv_bf16_takes_mfma(v.pattern, v.a) || (v.a.nvec <= kMaxFewVectors && gemv_bf16_takes_few(v.pattern, v.a));
}

// The small-result kernel wants both operands stored with k as the row index: a transposed A (K x M) and a
// row-major B (K x N).  A vector is that in either storage order: a 1 x K row is a K x 1 column with leading
// dimension 1.  Sets the leading dimensions the kernel is to use.
bool tall_storage(int transA, int transB, int64_t M, int64_t N, int64_t lda, int64_t ldb, int64_t *lda_t, int64_t *ldb_t)
{
    if (!(transA || M == 1) || !(!transB || N == 1)) return false;
    *lda_t = transA ? lda : 1;
    *ldb_t = !transB ? ldb : 1;
    return true;
}

// `split`: the call brings a workspace.
int plan_f32(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
             int64_t ldb, bool split, Plan *p, bool use_table = true)
{
    const Tuned *t = use_table ? find_tuned(0, transA, transB, M, N, K, split) : nullptr;
    bool vector = vector_call_f32(transA, transB, M, N, K, A, lda, B, ldb);
    if (vector && split && M > 8 && N > 8 && splitk_slices(M, N, K, 16) > 1) {
        // 9 .. 16 vectors against a matrix that is contiguous along k: a workgroup of that pattern fetches as many bytes of
        // vectors from the L2 as of matrix (16 x 8192 x 8192 103 - 155 us); the 64 x 64 tiles in K slices do it in 84 - 90.
        // Without a workspace the tiles take 270, and the other pattern streams at 3.2 - 3.6 TB/s either way (74 - 85 us).
        const VecMap v = vector_map(transA, transB, M, N, K, A, lda, B, ldb, nullptr, 1);
        vector = v.pattern == kVecCols;
    }
    SkinnyArgs sk;
    sk.K = (int)K;
    sk.parts = (int)(K / 256 < kSkinnyMaxParts ? K / 256 : kSkinnyMaxParts);
    if (!t && split && skinny_fits(M, N) && K >= 4096 && tall_storage(transA, transB, M, N, lda, ldb, &sk.lda, &sk.ldb) &&
        skinny_offsets_fit(sk)) {
        // a small result of long sums: one workgroup per 256 k (a row per lane) up to one per compute unit, each
        // with a partial result in the workspace; the pieces' lane offsets must fit, as the launcher checks them
        p->cfg = kF32_Skinny;
        p->slices = sk.parts;
    } else if (!t && vector) {
        const VecMap v = vector_map(transA, transB, M, N, K, A, lda, B, ldb, nullptr, 1);
        p->cfg = kF32_Vector;
        p->slices = split ? vector_slices(v.pattern, v.a.len, K, 32, v.a.nvec > 1 ? 16 : 4) : 1;
        // (several vectors against a matrix walked along k, up to 128 workgroups a slice: two workgroups per compute unit pay --
        // 8 x 2048 x 8192 against a transposed B 27 us in 2 slices, 24 in 4; 8 x 1024 x 16384 26 in 4, 24.6 in 8)
        if (split && v.a.nvec > 1 && v.pattern == kVecRows && ceil_div(v.a.len, 16) <= 128 && p->slices * 2 <= kMaxSlices && K / (p->slices * 2) >= 2048)
            p->slices *= 2;
        if (p->slices > 1 && (int64_t)p->slices * M * N * 4 > kMaxWorkspace) p->slices = (int)(kMaxWorkspace / (M * N * 4)) < 2 ? 1 : (int)(kMaxWorkspace / (M * N * 4));
    } else {
        p->slices = t ? t->slices : split ? splitk_slices(M, N, K, 16) : 1;
        if (!t && p->slices == 1 && use_table) t = find_tuned(0, transA, transB, M, N, K, false);
        unsigned main_fits = 0;
        for (int sh = 0; sh < kF32MainShapes; ++sh)
            main_fits |= (unsigned)f32_main_fits(sh, transA ? kMnContig : kKContig, transB ? kKContig : kMnContig, M, N, K, A, lda, B, ldb) << sh;
        if (t && t->tile >= kF32_Main && (!(main_fits >> (t->tile - kF32_Main) & 1) || !f32_main_slices_fit(K, t->slices))) t = nullptr;    // a row for operands aligned otherwise
        if (!t && split && main_fits) {
            // the direct-to-LDS shapes in K slices where that pays; otherwise the call is planned as one without a workspace
            const MainSplit ms = best_main_split(M, N, K, main_fits);
            p->slices = ms.slices;
            if (ms.slices > 1) {
                p->cfg = kF32_Main + ms.shape;
                return mode_f32(p->cfg, p->slices, M, N, K, A, lda, B, ldb, &p->mode);
            }
            if (use_table) t = find_tuned(0, transA, transB, M, N, K, false);
        }
        // a split runs on 64 x 64 tiles, or on 128 x 128 ones where those still give every compute unit a workgroup
        // and a slice keeps at least 1024 k (10-17 % faster there, measured on 256^2 ... 1024^2 with K up to 65536)
        // (not for a sliver under 128 rows or columns, part of whose 128-wide tile would be padding: 8 x 8192 x 8192 runs 57 %
        // faster on 64 x 64 tiles)
        const bool split128 = p->slices > 1 && ceil_div(M, 128) * ceil_div(N, 128) * p->slices >= 240 && K / p->slices >= 1024 && M >= 128 && N >= 128;
        int64_t one_cost = 0;
        p->cfg = t ? t->tile : p->slices > 1 ? (split128 ? kF32_128x128 : kF32_64x64) : tile_rule_f32(M, N, main_fits, &one_cost);
        // one launch leaves compute units idle in its last round: try two bands of direct-to-LDS shapes (tile times in
        // 0.1 ns per k; 4 us for the second launch); taken for a modelled gain of 3 % and more
        if (!t && p->slices == 1 && main_fits && (double)one_cost * 256.0 * 65536.0 > 1.03 * (double)M * (double)N * (double)kMainTileTime[0]) {
            const int a_lay = transA ? kMnContig : kKContig, b_lay = transB ? kKContig : kMnContig;
            const Bands b = best_bands(BandsKey{0, a_lay * 2 + b_lay, M, N, K, main_fits}, kF32MainShapes, [&](int sh, int64_t m, int64_t n) -> int64_t {
                if (!(main_fits >> sh & 1) || m < f32_main_tile_m(sh) || n < f32_main_tile_n(sh)) return -1;
                return ceil_div(ceil_div(m, f32_main_tile_m(sh)) * ceil_div(n, f32_main_tile_n(sh)), 256) * kMainTileTime[sh];
            }, 40000 / K);
            if (b.dim && b.cost * 100 <= one_cost * 97) {
                const float *A2 = A, *B2 = B;
                float *none = nullptr;
                shift_to_band(b.dim, b.at, a_lay, b_lay, A2, lda, B2, ldb, none, 0);
                const int64_t m1 = b.dim == 1 ? b.at : M, n1 = b.dim == 2 ? b.at : N;
                if (f32_main_fits(b.sh1, a_lay, b_lay, m1, n1, K, A, lda, B, ldb) &&
                    f32_main_fits(b.sh2, a_lay, b_lay, b.dim == 1 ? M - b.at : M, b.dim == 2 ? N - b.at : N, K, A2, lda, B2, ldb))
                    p->cfg = kF32_Main + b.sh1, p->cfg2 = kF32_Main + b.sh2, p->band_dim = b.dim, p->band_at = b.at;
            }
        }
    }
    return mode_f32(p->cfg, p->slices, M, N, K, A, lda, B, ldb, &p->mode);
}

// Tile rule for the bf16 direct-to-LDS kernel: the shape with the least modelled time.  A launch takes as many rounds
// as the compute unit with the most tiles, a round takes b ns per K-tile plus a ns around them (prologue, result
// written out), and -- unlike fp32 -- a last round that fills only part of the 256 compute units is shorter than a
// full one, down to three quarters: this kernel runs against the power limit, and with compute units idle the others
// clock higher.  b and a per shape are a least-squares fit to launches of every shape forced on 18 problems (4096^3 ...
// 10240^2 x 4096, 16384 x 4096 x 4096); on a second sweep of 22 problems the rule's choice was the measured winner or
// within 2 % of it on 20 (the others: 5 % on 7168^2 x 2048, 1.6 us on 4096^2 x 128).
// Returns the shape, or -1 when none fits the problem (fits: bit s set if shape s can take it).
constexpr int kBf16MainLarge = 6;        // the shapes this rule covers: those with a side of 256 or 192
constexpr int64_t kBf16MainPerKTile[kBf16MainLarge] = {1333, 1073, 780, 1037, 907, 808};      // in the order of the shapes
constexpr int64_t kBf16MainPerRound[kBf16MainLarge] = {8700, 5800, 4700, 7700, 3700, 5200};
int64_t bf16_main_cost(int sh, int64_t M, int64_t N, int64_t K)       // in 1/256 ns
{
    const int64_t tiles = ceil_div(M, bf16_main_tile_m(sh)) * ceil_div(N, bf16_main_tile_n(sh)), rest = tiles % 256;
    // (a launch that is one partial round gains less from its idle compute units than a last round behind full ones:
    // 192 tiles of 256 x 256 take 0.84 of a full round on 3072 x 4096 x 4096, 192 of 192 x 256 take 0.86 on 3072^3)
    const int64_t least = tiles < 256 ? 220 : 192;
    const int64_t rounds256 = tiles / 256 * 256 + (rest == 0 ? 0 : rest < least ? least : rest);       // in 1/256 of a round
    return rounds256 * (kBf16MainPerKTile[sh] * ceil_div(K, 64) + kBf16MainPerRound[sh]);
}
// The same for the 128 x 128 tile, in the same units: up to 256 tiles run one to a compute unit (450 ns per K-tile),
// beyond that two share a unit and its L2 path (780 ns: 2048^2 and 2048 x 4096 with K = 128 ... 8192); the time around
// the K-tiles is taken as that of the 128 x 256 shape, so that a short K does not decide between the two by it.
int64_t bf16_main128_cost(int64_t M, int64_t N, int64_t K)
{
    const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 128), nk = ceil_div(K, 64), rest = tiles % 512;
    const int64_t one = 450 * nk + 4700, two = 780 * nk + 5400;
    return tiles / 512 * 256 * two + (rest == 0 ? 0 : rest <= 256 ? (rest < 220 ? 220 : rest) * one : 256 * two);
}
int tile_rule_bf16_main(int64_t M, int64_t N, int64_t K, unsigned fits, int64_t *cost_out = nullptr)
{
    int best = -1;
    int64_t best_cost = 0;
    for (int sh = 0; sh < kBf16MainLarge; ++sh) {
        if (!(fits >> sh & 1)) continue;
        const int64_t cost = bf16_main_cost(sh, M, N, K);
        if (best < 0 || cost < best_cost) best = sh, best_cost = cost;
    }
    if (cost_out) *cost_out = best_cost;
    return best;
}

// K slices for bf16 problems of 64 rows and columns and more that bring a workspace: the general kernel's 64 x 64 tile or,
// where it fits, the direct-to-LDS kernel's 128 x 128 tile, in the slice count with the least modelled time.  Per K-tile of
// 64 and workgroup: 64 x 64 248 ns alone on a compute unit, 208 ns each with several (half as much again when an operand
// is contiguous along m / n, which that kernel regroups in registers); 128 x 128 450 ns alone, 780 ns for two; around the K
// loop 3.4 / 4.7 us; for slices the second launch (4 us + 0.15 us per slice) and its traffic (slices + 1 results at 3 TB/s); a slice keeps 512 k
// or more.  Measured against the rule this replaced (about 1024 workgroups): 256^2 x 16384 26 -> 17 us, 256^2 x 8192
// 17 -> 11, 128 x 2048 x 4096 15 -> 9, 1536 x 1024 x 8192 55 -> 46.  Costs in ns.
struct Bf16Split {
    int cfg = kBf16_64x64, slices = 1;
    int64_t cost = 0;
};
Bf16Split best_bf16_split(int64_t M, int64_t N, int64_t K, bool main128_fits, bool k_contiguous)
{
    Bf16Split best, unsplit;
    bool have = false, have_unsplit = false;
    const int64_t nk = ceil_div(K, 64), t64 = ceil_div(M, 64) * ceil_div(N, 64), t128 = ceil_div(M, 128) * ceil_div(N, 128);
    for (int kind = 0; kind < (main128_fits ? 2 : 1); ++kind) {
        for (int sl = 1; sl <= kMaxSlices; ++sl) {
            if (sl > 1 && (int64_t)sl * M * N * 4 > kMaxWorkspace) break;
            const int64_t len = ceil_div(nk, sl);               // K-tiles per slice
            if (sl > 1 && (len < 8 || (sl - 1) * len >= nk || (kind == 1 && !bf16_main_slices_fit(K, sl)))) continue;
            int64_t cost;
            if (kind == 0) {
                // (its workgroups drift apart along K, and once the operand panels of a slice outgrow 8.75 MB they no longer
                // meet in the L2: 1024^2 x 2048, 8.4 MB, runs 0.23 us per K-tile, 768^2 x 3072, 9.0 MB, 0.43)
                // (slices that run side by side help only in part: 7 / 5 when the whole problem's panels outgrow that size)
                const int64_t limit = (int64_t)35 << 18, w = ceil_div(t64 * sl, 256);
                const int64_t slow = (M + N) * len * 128 > limit ? 9 : (M + N) * nk * 128 > limit ? 7 : 5;
                cost = w * len * (w == 1 ? 248 : 208) * (k_contiguous ? 2 : 3) / 2 * slow / 5 + 3400;
            } else {
                const int64_t groups = t128 * sl, rest = groups % 512;
                cost = (groups / 512 + (rest > 256)) * len * 780 + (rest > 0 && rest <= 256) * len * 450 + 4700;
            }
            if (sl > 1) cost += 4000 + sl * 150 + (sl + 1) * M * N * 4 / 3000;
            const int cfg = kind == 0 ? (int)kBf16_64x64 : bf16_main_candidate(kBf16MainLarge);
            if (sl == 1 && (!have_unsplit || cost < unsplit.cost)) unsplit.cfg = cfg, unsplit.slices = 1, unsplit.cost = cost, have_unsplit = true;
            if (!have || cost < best.cost) best.cfg = cfg, best.slices = sl, best.cost = cost, have = true;
        }
    }
    return best.slices > 1 && best.cost * 100 > unsplit.cost * 95 ? unsplit : best;
}

int mode_bf16(int cfg, int slices, int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda, const uint16_t *B,
              int64_t ldb, int *mode)
{
    *mode = 0;
    if (bf16_main_shape(cfg) >= 0) return FSRGEMM_OK;       // whether it fits the problem is its own check
    const int b = kBf16Tile[cfg];
    if (ceil_div(M, b) * ceil_div(N, b) * slices >= ((int64_t)1 << 31)) return FSRGEMM_ERR_INVALID_ARG;
    const bool vec = aligned16(A) && aligned16(B) && lda % 8 == 0 && ldb % 8 == 0;
    *mode = !vec ? kScalar : (M >= b && N >= b && K % 64 == 0 && K > 0) ? kFast : kVecPred;
    return FSRGEMM_OK;
}

int plan_bf16(int a_lay, int b_lay, int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda, const uint16_t *B,
              int64_t ldb, bool split, Plan *p, bool use_table = true)
{
    const int transA = a_lay == kMnContig, transB = b_lay == kKContig;
    const Tuned *t = use_table ? find_tuned(1, transA, transB, M, N, K, split) : nullptr;
    // With 5 .. 8 vectors the widening and the multiply-adds of the streaming kernels occupy the vector units (2.6 - 2.9 TB/s
    // on 8 x 8192 x 8192); where a workspace lets the 64 x 64 tiles split K they stream faster (26 - 34 us against 35 - 46), so
    // such calls stay with the tiles.  Without a workspace, and up to 4 vectors either way, the streaming kernels win (plain
    // 8 x 8192 x 8192 46 - 81 us against 78 - 140; 4 x 8192 x 8192 36 - 53 against 78 - 411).
    // The matrix-core kernels (up to 16 vectors contiguous along k against a matrix contiguous along k) run 16 x 8192 x 8192
    // in 31 us without a workspace against the tiles' 79, 8 x ... in 27.5, 2 x ... in 23; with a workspace the tiles' split is
    // level or ahead on long matrices with more than 8 vectors (16 x 8192 x 8192 26 us against 29, 16 x 28672 x 8192 100 - 113
    // against 108), not on short ones (12 x 1024 x 16384: 13 us in 8 slices against 20).
    const bool tiles_can_split = split && (K >= 3072 || M < 64 || N < 64) && splitk_slices(M, N, K, 64) > 1;
    bool vector = !t && vector_call_bf16(transA, transB, M, N, K, A, lda, B, ldb);
    if (vector && !vector_shape(M, N, K) && tiles_can_split) {
        const VecMap16 v = vector_map16(transA, transB, M, N, K, A, lda, B, ldb, nullptr, 1);
        vector = gemv_bf16_takes_mfma(v.pattern, v.a) ? v.a.nvec <= 8 || v.a.len < 8192 : v.a.nvec <= 4;
    }
    if (vector) {
        const VecMap16 v = vector_map16(transA, transB, M, N, K, A, lda, B, ldb, nullptr, 1);
        p->cfg = kBf16_Vector;
        // (matrix rows per workgroup: 4 with one vector, 16 with several, 32 in the matrix-core kernel that stages the vectors in LDS)
        const int rows_per_group = v.a.nvec == 1 ? 4 : gemv_bf16_takes_mfma(v.pattern, v.a) && v.a.nvec > kMfmaDirectVectors ? 32 : 16;
        p->slices = split ? vector_slices(v.pattern, v.a.len, K, 64, rows_per_group) : 1;
        if (p->slices > 1 && (int64_t)p->slices * M * N * 4 > kMaxWorkspace) p->slices = (int)(kMaxWorkspace / (M * N * 4)) < 2 ? 1 : (int)(kMaxWorkspace / (M * N * 4));
        p->mode = 0;
        return ceil_div(M > N ? M : N, 4) * p->slices >= ((int64_t)1 << 31) ? FSRGEMM_ERR_INVALID_ARG : FSRGEMM_OK;
    }
    unsigned main_fits = 0;
    for (int sh = 0; sh < kBf16MainShapes; ++sh) main_fits |= (unsigned)bf16_main_fits(sh, a_lay, b_lay, M, N, K, A, lda, B, ldb) << sh;
    // (Under 128 rows or columns the earlier rule stays: about 1024 workgroups of the general kernel.  Its tiles get through
    // a short K quickly enough that a second launch costs more than the split gains -- on 256^2 ... 1024^2 splits lost 5-80 %
    // with K up to 2560 -- except for a sliver under 64 rows or columns, which runs on checked loads and gains at any K the
    // rule cuts: 16 x 8192 x 2048 23 -> 12 us.)
    const bool narrow = M < 128 || N < 128;
    p->slices = t ? t->slices : split && narrow && (K >= 3072 || M < 64 || N < 64) ? splitk_slices(M, N, K, 64) : 1;
    if (!t && split && !narrow && ceil_div(M, 256) * ceil_div(N, 256) < 128) {
        // the modelled best of 64 x 64 general tiles and 128 x 128 direct-to-LDS tiles in slices; an unsplit winner leaves
        // the call to the rules for calls without a workspace
        const Bf16Split bs = best_bf16_split(M, N, K, (main_fits >> kBf16MainLarge & 1) != 0, a_lay == kKContig && b_lay == kKContig);
        if (bs.slices > 1) {
            p->cfg = bs.cfg, p->slices = bs.slices;
            return mode_bf16(p->cfg, p->slices, M, N, K, A, lda, B, ldb, &p->mode);
        }
    }
    if (!t && p->slices == 1 && use_table) t = find_tuned(1, transA, transB, M, N, K, false);
    if (t && bf16_main_shape(t->tile) >= 0 && (!(main_fits >> bf16_main_shape(t->tile) & 1) || !bf16_main_slices_fit(K, t->slices))) t = nullptr;  // a row for operands aligned otherwise
    if (t) p->cfg = t->tile;
    // a split runs on 128 x 128 tiles where those still give every compute unit a workgroup (up to 30 % faster than
    // 64 x 64 ones there, measured on 256^2 ... 1024^2 with K up to 65536), else on 64 x 64 tiles
    // (and, as for fp32, not for a sliver most of whose 128-wide tile would be padding: 32 x 28672 x 8192 takes 0.129 ms on
    // 128 x 128 tiles and 0.121 on 64 x 64 ones, 96 x 8192 x 8192 0.047 and 0.039)
    else if (p->slices > 1) p->cfg = ceil_div(M, 128) * ceil_div(N, 128) * p->slices >= 240 && M >= 128 && N >= 128 ? kBf16_128x128 : kBf16_64x64;
    // where 256 x 256 tiles give at least half the compute units one each: the direct-to-LDS kernel in the shape that
    // fills whole rounds, or, where it does not fit (alignment, a K that is not whole 16-byte pieces), the general
    // kernel of that tile
    else if (ceil_div(M, 256) * ceil_div(N, 256) >= 128) {
        int64_t one_cost = 0;
        main_fits &= (1u << kBf16MainLarge) - 1;        // the shapes the cost rule covers
        p->cfg = main_fits ? bf16_main_candidate(tile_rule_bf16_main(M, N, K, main_fits, &one_cost)) : (int)kBf16_256x256;
        // two bands, as for fp32 (costs in 1/256 ns; 4 us for the second launch; taken for a modelled gain of 4 % and more)
        // (not where the one launch is within 3 % of 256 x 256 tiles in whole rounds, the best any plan can do)
        if (main_fits && (double)one_cost * 65536.0 > 1.03 * (double)M * (double)N * (double)(kBf16MainPerKTile[0] * ceil_div(K, 64) + kBf16MainPerRound[0])) {
            const Bands b = best_bands(BandsKey{1, a_lay * 2 + b_lay, M, N, K, main_fits}, kBf16MainLarge, [&](int sh, int64_t m, int64_t n) -> int64_t {
                if (!(main_fits >> sh & 1) || m < bf16_main_tile_m(sh) || n < bf16_main_tile_n(sh)) return -1;
                return bf16_main_cost(sh, m, n, K);
            }, (int64_t)4000 * 256);
            if (b.dim && b.cost * 100 <= one_cost * 96) {
                const uint16_t *A2 = A, *B2 = B;
                float *none = nullptr;
                shift_to_band(b.dim, b.at, a_lay, b_lay, A2, lda, B2, ldb, none, 0);
                if (bf16_main_fits(b.sh1, a_lay, b_lay, b.dim == 1 ? b.at : M, b.dim == 2 ? b.at : N, K, A, lda, B, ldb) &&
                    bf16_main_fits(b.sh2, a_lay, b_lay, b.dim == 1 ? M - b.at : M, b.dim == 2 ? N - b.at : N, K, A2, lda, B2, ldb))
                    p->cfg = bf16_main_candidate(b.sh1), p->cfg2 = bf16_main_candidate(b.sh2), p->band_dim = b.dim, p->band_at = b.at;
            }
        }
    }
    // smaller problems: the direct-to-LDS kernel's 128 x 128 tile where it fits and gives three quarters of the compute
    // units a workgroup (up to two share a unit; 2048^3 653 -> 807 TFLOP/s, 1024 x 4096 x 4096 771 -> 973, 1536 x 2048^2
    // 542 -> 581 against the general tiles; with 144 tiles, 1536^3, it is level with the general 64 x 64 tile), else the
    // general kernel's 128 x 128 tile where that fills the units, else its 64 x 64 tile
    // (with an operand contiguous along m / n the general kernel stages through registers and is slower: there the
    // 128 x 128 tile wins from 4 tiles on -- level at 256^3 and 512^3, 768^3 83-105 -> 107-112, 1024^3 156-198 -> 212-222,
    // 1536^3 194-290 -> 392-405, 256^2 x 65536 0.69-0.87 -> 0.59-0.60 ms)
    // (from 128 tiles on when K is 2048 or longer and the problem has 512 rows and columns: 1536^2 x 8192 80 -> 71 us, x 16384
    // 159 -> 147, level at K = 1536)
    else if ((main_fits >> kBf16MainLarge & 1) &&
             ceil_div(M, 128) * ceil_div(N, 128) >= (a_lay == kKContig && b_lay == kKContig ? (K >= 2048 && M >= 512 && N >= 512 ? 128 : 192) : 4)) {
        p->cfg = bf16_main_candidate(kBf16MainLarge);
        // between 64 and 127 tiles of 256 x 256 a larger shape in one round can beat two 128 x 128 tiles to a compute unit
        // (2048 x 2560 x 8192 852 -> 956 TFLOP/s on 128 x 256, 1792 x 4096 x 4096 1022 -> 1063): by the modelled times, where
        // K is long enough for them to be about the K-tiles (with K = 256 the shapes' fitted constants would decide)
        if (ceil_div(M, 256) * ceil_div(N, 256) >= 64 && K >= 1024) {
            int64_t cost = 0;
            const int sh = tile_rule_bf16_main(M, N, K, main_fits & ((1u << kBf16MainLarge) - 1), &cost);
            if (sh >= 0 && cost < bf16_main128_cost(M, N, K)) p->cfg = bf16_main_candidate(sh);
        }
    }
    else if (ceil_div(M, 128) * ceil_div(N, 128) >= 256) p->cfg = kBf16_128x128;
    else p->cfg = kBf16_64x64;
    if (p->cfg == kBf16_Vector) {       // a row of the selection table
        p->mode = 0;
        return vector_call_bf16(transA, transB, M, N, K, A, lda, B, ldb) ? FSRGEMM_OK : FSRGEMM_ERR_INVALID_ARG;
    }
    return mode_bf16(p->cfg, p->slices, M, N, K, A, lda, B, ldb, &p->mode);
}

// gfx950 check for the current device, cached per device ordinal (racing first calls just repeat the query).
int device_ok()
{
    constexpr int kMaxDev = 64;
    static std::atomic<int> cache[kMaxDev];     // 0 = unknown, 1 = gfx950, 2 = something else
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return FSRGEMM_ERR_UNSUPPORTED_DEVICE;
    const bool cached = dev >= 0 && dev < kMaxDev;
    if (cached) {
        const int c = cache[dev].load(std::memory_order_relaxed);
        if (c) return c == 1 ? FSRGEMM_OK : FSRGEMM_ERR_UNSUPPORTED_DEVICE;
    }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return FSRGEMM_ERR_UNSUPPORTED_DEVICE;
    const bool ok = strncmp(prop.gcnArchName, "gfx950", 6) == 0;
    if (cached) cache[dev].store(ok ? 1 : 2, std::memory_order_relaxed);
    return ok ? FSRGEMM_OK : FSRGEMM_ERR_UNSUPPORTED_DEVICE;
}

GemmArgs pack(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb, float *C,
              int64_t ldc)
{
    GemmArgs a;
    a.M = (int)M;
    a.N = (int)N;
    a.K = (int)K;
    a.A = A;
    a.lda = lda;
    a.B = B;
    a.ldb = ldb;
    a.C = C;
    a.ldc = ldc;
    a.k_slices = 1;
    a.slice_stride = 0;
    return a;
}

}  // namespace

namespace fsrgemm {

hipError_t ensure_dynamic_lds(const void *kernel, int bytes, std::atomic<uint64_t> &done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < 64;
    const uint64_t bit = tracked ? (uint64_t)1 << dev : 0;
    if (tracked && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && tracked) done.fetch_or(bit, std::memory_order_release);
    return e;
}

}  // namespace fsrgemm

namespace {

// Launch of a planned product: in one piece into C, or (p.slices > 1) as partial products into the workspace
// followed by the kernel that adds the slices in slice order.
int run_f32(const Plan &p, int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
            const float *B, int64_t ldb, float *C, int64_t ldc, float *ws, hipStream_t s)
{
    const int rc = device_ok();
    if (rc != FSRGEMM_OK) return rc;
    if (p.cfg == kF32_Skinny) {
        SkinnyArgs a;
        a.A = A, a.B = B;
        if (!tall_storage(transA, transB, M, N, lda, ldb, &a.lda, &a.ldb)) return FSRGEMM_ERR_INVALID_ARG;
        a.M = (int)M, a.N = (int)N, a.K = (int)K, a.parts = p.slices, a.partial = ws;
        return launch_skinny_f32(a, C, ldc, s) == hipSuccess ? FSRGEMM_OK : FSRGEMM_ERR_LAUNCH;
    }
    const bool split = p.slices > 1;
    hipError_t e;
    if (p.cfg >= kF32_Main) {
        const int a_lay = transA ? kMnContig : kKContig, b_lay = transB ? kKContig : kMnContig;
        if (split) {        // partial products of the K slices into the workspace, then their sum in slice order
            if (p.band_dim != 0) return FSRGEMM_ERR_INVALID_ARG;        // the planners never pair the two
            GemmArgs a = pack(M, N, K, A, lda, B, ldb, ws, N);
            a.k_slices = p.slices;
            a.slice_stride = M * N;
            e = launch_f32_main(p.cfg - kF32_Main, a_lay, b_lay, a, s);
            if (e == hipSuccess) e = launch_splitk_reduce(ws, p.slices, M * N, C, (int)M, (int)N, ldc, s);
        } else if (p.band_dim == 0) {
            e = launch_f32_main(p.cfg - kF32_Main, a_lay, b_lay, pack(M, N, K, A, lda, B, ldb, C, ldc), s);
        } else {
            const int64_t m1 = p.band_dim == 1 ? p.band_at : M, n1 = p.band_dim == 2 ? p.band_at : N;
            e = launch_f32_main(p.cfg - kF32_Main, a_lay, b_lay, pack(m1, n1, K, A, lda, B, ldb, C, ldc), s);
            if (e == hipSuccess) {
                shift_to_band(p.band_dim, p.band_at, a_lay, b_lay, A, lda, B, ldb, C, ldc);
                e = launch_f32_main(p.cfg2 - kF32_Main, a_lay, b_lay, pack(p.band_dim == 1 ? M - m1 : M, p.band_dim == 2 ? N - n1 : N, K, A, lda, B, ldb, C, ldc), s);
            }
        }
        return e == hipSuccess ? FSRGEMM_OK : e == hipErrorInvalidValue ? FSRGEMM_ERR_INVALID_ARG : FSRGEMM_ERR_LAUNCH;
    }
    if (p.cfg == kF32_Vector) {
        VecMap v = vector_map(transA, transB, M, N, K, A, lda, B, ldb, C, ldc);
        if (split) {        // a slice of the workspace is an M x N matrix with rows of N
            v.a.y = ws, v.a.k_slices = p.slices, v.a.slice_stride = M * N;
            if (N <= M) v.a.incy = N, v.a.ldy = 1;
            else v.a.incy = 1, v.a.ldy = N;
        }
        e = launch_gemv_f32(v.pattern, v.a, s);
    } else {
        GemmArgs a = pack(M, N, K, A, lda, B, ldb, split ? ws : C, split ? N : ldc);
        a.k_slices = p.slices;
        a.slice_stride = split ? M * N : 0;
        e = launch_f32(p.cfg, p.mode, transA ? kMnContig : kKContig, transB ? kKContig : kMnContig, a, s);
    }
    if (e == hipSuccess && split) e = launch_splitk_reduce(ws, p.slices, M * N, C, (int)M, (int)N, ldc, s);
    return e == hipSuccess ? FSRGEMM_OK : FSRGEMM_ERR_LAUNCH;
}

int run_bf16(const Plan &p, int a_lay, int b_lay, int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda,
             const uint16_t *B, int64_t ldb, float *C, int64_t ldc, float *ws, hipStream_t s)
{
    const bool split = p.slices > 1;
    const int rc = device_ok();
    if (rc != FSRGEMM_OK) return rc;
    hipError_t e;
    if (bf16_main_shape(p.cfg) >= 0) {
        if (split) {        // partial products of the K slices into the workspace, then their sum in slice order
            if (p.band_dim != 0) return FSRGEMM_ERR_INVALID_ARG;        // the planners never pair the two
            GemmArgs a = pack(M, N, K, A, lda, B, ldb, ws, N);
            a.k_slices = p.slices;
            a.slice_stride = M * N;
            e = launch_bf16_main(bf16_main_shape(p.cfg), a_lay, b_lay, a, s);
            if (e == hipSuccess) e = launch_splitk_reduce(ws, p.slices, M * N, C, (int)M, (int)N, ldc, s);
        } else if (p.band_dim == 0) {
            e = launch_bf16_main(bf16_main_shape(p.cfg), a_lay, b_lay, pack(M, N, K, A, lda, B, ldb, C, ldc), s);
        } else {
            const int64_t m1 = p.band_dim == 1 ? p.band_at : M, n1 = p.band_dim == 2 ? p.band_at : N;
            e = launch_bf16_main(bf16_main_shape(p.cfg), a_lay, b_lay, pack(m1, n1, K, A, lda, B, ldb, C, ldc), s);
            if (e == hipSuccess) {
                shift_to_band(p.band_dim, p.band_at, a_lay, b_lay, A, lda, B, ldb, C, ldc);
                e = launch_bf16_main(bf16_main_shape(p.cfg2), a_lay, b_lay, pack(p.band_dim == 1 ? M - m1 : M, p.band_dim == 2 ? N - n1 : N, K, A, lda, B, ldb, C, ldc), s);
            }
        }
        return e == hipSuccess ? FSRGEMM_OK : e == hipErrorInvalidValue ? FSRGEMM_ERR_INVALID_ARG : FSRGEMM_ERR_LAUNCH;
    }
    if (p.cfg == kBf16_Vector) {
        VecMap16 v = vector_map16(a_lay == kMnContig, b_lay == kKContig, M, N, K, A, lda, B, ldb, C, ldc);
        if (split) {        // a slice of the workspace is an M x N matrix with rows of N
            v.a.y = ws, v.a.k_slices = p.slices, v.a.slice_stride = M * N;
            if (N <= M) v.a.incy = N, v.a.ldy = 1;
            else v.a.incy = 1, v.a.ldy = N;
        }
        e = launch_gemv_bf16(v.pattern, v.a, s);
    } else {
        GemmArgs a = pack(M, N, K, A, lda, B, ldb, split ? ws : C, split ? N : ldc);
        a.k_slices = p.slices;
        a.slice_stride = split ? M * N : 0;
        e = launch_bf16(p.cfg, p.mode, a_lay, b_lay, a, s);
    }
    if (e == hipSuccess && split) e = launch_splitk_reduce(ws, p.slices, M * N, C, (int)M, (int)N, ldc, s);
    return e == hipSuccess ? FSRGEMM_OK : FSRGEMM_ERR_LAUNCH;
}

// Scratch memory of gemm_f32_noalloc: one array per device that holds the library, there until the process ends.
// In host code the array's name is not a device address: the address is looked up once per device, with that device
// current, and only that pointer is handed to kernels.
constexpr int64_t kStaticScratchBytes = FSRGEMM_NOALLOC_SCRATCH_BYTES;
static_assert(kStaticScratchBytes >= kMaxWorkspace, "every split the planner makes fits the array");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

int static_scratch(float **out)
{
    constexpr int kMaxDev = 64;
    static std::atomic<void *> known[kMaxDev];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return FSRGEMM_ERR_UNSUPPORTED_DEVICE;
    const bool cached = dev >= 0 && dev < kMaxDev;
    void *ptr = cached ? known[dev].load(std::memory_order_acquire) : nullptr;
    if (ptr == nullptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return FSRGEMM_ERR_LAUNCH;
        if (cached) known[dev].store(ptr, std::memory_order_release);
    }
    *out = static_cast<float *>(ptr);
    return FSRGEMM_OK;
}

// "first kernel + second kernel (rows | columns from <cut>)" of a product that runs as two bands; the text lives in a
// buffer of the calling thread until its next such query
const char *two_band_name(const Plan &p, const char *first, const char *second)
{
    static thread_local char text[192];
    snprintf(text, sizeof text, "%s + %s (%s from %lld)", first, second, p.band_dim == 1 ? "rows" : "columns", (long long)p.band_at);
    return text;
}

bool extents_ok(int64_t M, int64_t N, int64_t K)
{
    const int64_t lim = (int64_t)1 << 31;
    return M >= 0 && N >= 0 && K >= 0 && M < lim && N < lim && K < lim;
}

// a workspace a split can use: big enough and aligned for a float
bool workspace_fits(const void *workspace, int64_t bytes, int slices, int64_t M, int64_t N)
{
    return workspace != nullptr && bytes >= (int64_t)slices * M * N * 4 && (reinterpret_cast<uintptr_t>(workspace) & 3u) == 0;
}

// Checks of a forced configuration that do not depend on the precision: the slice count, and for a split the
// workspace and a K range that gives every slice at least one K-tile.
bool forced_ok(int tile, int tile_count, int slices, int64_t M, int64_t N, int64_t K, int k_tile, const void *workspace,
               int64_t workspace_bytes)
{
    if (tile < 0 || tile >= tile_count || slices < 1 || slices > kMaxSlices) return false;
    if (workspace_bytes < 0 || (workspace_bytes > 0 && workspace == nullptr)) return false;
    if (slices == 1) return true;
    return M > 0 && N > 0 && slices <= ceil_div(K, k_tile) && (int64_t)slices * M * N * 4 <= kMaxWorkspace &&
           workspace_fits(workspace, workspace_bytes, slices, M, N);
}

}  // namespace

extern "C" {

int gemm_f32(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb, float *C,
             int64_t ldc, void *stream)
{
    return gemm_f32_ex(0, 0, M, N, K, A, lda, B, ldb, C, ldc, stream);
}

int gemm_f32_ex(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                int64_t ldb, float *C, int64_t ldc, void *stream)
{
    return gemm_f32_ws(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, nullptr, 0, stream);
}

int gemm_f32_noalloc(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                     int64_t ldb, float *C, int64_t ldc, void *stream)
{
    int rc = check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc);
    if (rc != FSRGEMM_OK) return rc;
    Plan p;
    rc = plan_f32(transA, transB, M, N, K, A, lda, B, ldb, true, &p);
    if (rc != FSRGEMM_OK) return rc;
    const bool needs = p.slices > 1 || p.cfg == kF32_Skinny;
    if (needs && (int64_t)p.slices * M * N * 4 > kStaticScratchBytes) return FSRGEMM_ERR_SCRATCH_LIMIT;
    if (M == 0 || N == 0) return FSRGEMM_OK;
    float *ws = nullptr;
    if (needs) {
        rc = static_scratch(&ws);
        if (rc != FSRGEMM_OK) return rc;
    }
    return run_f32(p, transA, transB, M, N, K, A, lda, B, ldb, C, ldc, ws, static_cast<hipStream_t>(stream));
}

int64_t gemm_f32_workspace_bytes(int transA, int transB, int64_t M, int64_t N, int64_t K)
{
    if (!extents_ok(M, N, K)) return 0;
    // The slices depend on whether the operands' alignment lets the direct-to-LDS kernel run, which the query cannot
    // know: the larger of the two plans' workspaces serves either.
    int64_t bytes = 0;
    for (const float *fake : {static_cast<const float *>(nullptr), reinterpret_cast<const float *>(uintptr_t{4})}) {
        Plan p;
        if (plan_f32(transA, transB, M, N, K, fake, 4, fake, 4, true, &p) != FSRGEMM_OK) continue;
        const int64_t need = p.slices > 1 || p.cfg == kF32_Skinny ? (int64_t)p.slices * M * N * 4 : 0;
        if (need > bytes) bytes = need;
    }
    return bytes;
}

int gemm_f32_ws(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                int64_t ldb, float *C, int64_t ldc, void *workspace, int64_t workspace_bytes, void *stream)
{
    int rc = check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc);
    if (rc != FSRGEMM_OK) return rc;
    if (workspace_bytes < 0 || (workspace_bytes > 0 && workspace == nullptr)) return FSRGEMM_ERR_INVALID_ARG;
    Plan p;
    rc = plan_f32(transA, transB, M, N, K, A, lda, B, ldb, workspace != nullptr, &p);
    if (rc == FSRGEMM_OK && (p.slices > 1 || p.cfg == kF32_Skinny) && !workspace_fits(workspace, workspace_bytes, p.slices, M, N))
        rc = plan_f32(transA, transB, M, N, K, A, lda, B, ldb, false, &p);
    if (rc != FSRGEMM_OK) return rc;
    if (M == 0 || N == 0) return FSRGEMM_OK;
    return run_f32(p, transA, transB, M, N, K, A, lda, B, ldb, C, ldc, static_cast<float *>(workspace),
                   static_cast<hipStream_t>(stream));
}

int gemm_f32_cfg(int tile, int k_slices, int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A,
                 int64_t lda, const float *B, int64_t ldb, float *C, int64_t ldc, void *workspace, int64_t workspace_bytes,
                 void *stream)
{
    int rc = check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc);
    if (rc != FSRGEMM_OK) return rc;
    if (tile == kF32_Skinny) {      // its k_slices are workgroups with a partial result each: up to 256, and a workspace even for one
        if (M == 0 || N == 0) return FSRGEMM_OK;
        SkinnyArgs probe;
        if (!tall_storage(transA, transB, M, N, lda, ldb, &probe.lda, &probe.ldb) || !skinny_fits(M, N) || K < 1 || k_slices < 1 ||
            k_slices > kSkinnyMaxParts || k_slices > K || workspace_bytes < 0 || !workspace_fits(workspace, workspace_bytes, k_slices, M, N))
            return FSRGEMM_ERR_INVALID_ARG;
        probe.K = (int)K, probe.parts = k_slices;
        if (!skinny_offsets_fit(probe)) return FSRGEMM_ERR_INVALID_ARG;
    } else if (tile >= kF32_Main && tile < kF32_Main + kF32MainShapes) {     // only problems it fits; slices of whole K-tiles
        if (!forced_ok(tile, kF32_Main + kF32MainShapes, k_slices, M, N, K, 32, workspace, workspace_bytes)) return FSRGEMM_ERR_INVALID_ARG;
        if (M == 0 || N == 0) return FSRGEMM_OK;
        if (!f32_main_fits(tile - kF32_Main, transA ? kMnContig : kKContig, transB ? kKContig : kMnContig, M, N, K, A, lda, B, ldb) ||
            !f32_main_slices_fit(K, k_slices))
            return FSRGEMM_ERR_INVALID_ARG;
    } else {
        if (!forced_ok(tile, kF32_Vector + 1, k_slices, M, N, K, 16, workspace, workspace_bytes)) return FSRGEMM_ERR_INVALID_ARG;
        if (tile == kF32_Vector && !vector_call_f32(transA, transB, M, N, K, A, lda, B, ldb) && M > 0 && N > 0) return FSRGEMM_ERR_INVALID_ARG;
    }
    Plan p = {tile, 0, k_slices};
    rc = mode_f32(tile, k_slices, M, N, K, A, lda, B, ldb, &p.mode);
    if (rc != FSRGEMM_OK) return rc;
    if (M == 0 || N == 0) return FSRGEMM_OK;
    return run_f32(p, transA, transB, M, N, K, A, lda, B, ldb, C, ldc, static_cast<float *>(workspace),
                   static_cast<hipStream_t>(stream));
}

int fsrgemm_plan_f32(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                     int64_t ldb, int flags, int *tile, int *k_slices)
{
    if (!extents_ok(M, N, K) || tile == nullptr || k_slices == nullptr || (flags & ~3)) return FSRGEMM_ERR_INVALID_ARG;
    Plan p;
    const int rc = plan_f32(transA, transB, M, N, K, A, lda, B, ldb, (flags & 1) != 0, &p, (flags & 2) == 0);
    if (rc != FSRGEMM_OK) return rc;
    *tile = p.cfg;
    *k_slices = p.slices;
    return FSRGEMM_OK;
}

int fsrgemm_tile_count_f32(void) { return kF32_Main + kF32MainShapes; }

int fsrgemm_bands_f32(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                      int64_t ldb, int flags, int *dim, int64_t *at, int *tile_first, int *tile_second)
{
    if (!extents_ok(M, N, K) || dim == nullptr || at == nullptr || tile_first == nullptr || tile_second == nullptr || (flags & ~3)) return FSRGEMM_ERR_INVALID_ARG;
    Plan p;
    const int rc = plan_f32(transA, transB, M, N, K, A, lda, B, ldb, (flags & 1) != 0, &p, (flags & 2) == 0);
    if (rc != FSRGEMM_OK) return rc;
    *dim = p.band_dim, *at = p.band_at, *tile_first = p.cfg, *tile_second = p.band_dim ? p.cfg2 : p.cfg;
    return FSRGEMM_OK;
}

int gemm_bf16(int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
              float *C, int64_t ldc, void *stream)
{
    return gemm_bf16_ex(0, 1, M, N, K, A, lda, B, ldb, C, ldc, stream);
}

int gemm_bf16_ex(int transA, int transB, int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda,
                 const uint16_t *B, int64_t ldb, float *C, int64_t ldc, void *stream)
{
    return gemm_bf16_ws(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, nullptr, 0, stream);
}

int64_t gemm_bf16_workspace_bytes(int transA, int transB, int64_t M, int64_t N, int64_t K)
{
    if (!extents_ok(M, N, K)) return 0;
    // as for fp32: the larger of the plans for operands the direct-to-LDS kernel can and cannot take
    int64_t bytes = 0;
    for (const uint16_t *fake : {static_cast<const uint16_t *>(nullptr), reinterpret_cast<const uint16_t *>(uintptr_t{2})}) {
        Plan p;
        if (plan_bf16(transA ? kMnContig : kKContig, transB ? kKContig : kMnContig, M, N, K, fake, 8, fake, 8, true, &p) != FSRGEMM_OK) continue;
        const int64_t need = p.slices > 1 ? (int64_t)p.slices * M * N * 4 : 0;
        if (need > bytes) bytes = need;
    }
    return bytes;
}

int gemm_bf16_ws(int transA, int transB, int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda,
                 const uint16_t *B, int64_t ldb, float *C, int64_t ldc, void *workspace, int64_t workspace_bytes,
                 void *stream)
{
    int rc = check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc);
    if (rc != FSRGEMM_OK) return rc;
    if (workspace_bytes < 0 || (workspace_bytes > 0 && workspace == nullptr)) return FSRGEMM_ERR_INVALID_ARG;
    const int a_lay = transA ? kMnContig : kKContig, b_lay = transB ? kKContig : kMnContig;
    Plan p;
    rc = plan_bf16(a_lay, b_lay, M, N, K, A, lda, B, ldb, workspace != nullptr, &p);
    if (rc == FSRGEMM_OK && p.slices > 1 && !workspace_fits(workspace, workspace_bytes, p.slices, M, N))
        rc = plan_bf16(a_lay, b_lay, M, N, K, A, lda, B, ldb, false, &p);
    if (rc != FSRGEMM_OK) return rc;
    if (M == 0 || N == 0) return FSRGEMM_OK;
    return run_bf16(p, a_lay, b_lay, M, N, K, A, lda, B, ldb, C, ldc, static_cast<float *>(workspace),
                    static_cast<hipStream_t>(stream));
}

int gemm_bf16_cfg(int tile, int k_slices, int transA, int transB, int64_t M, int64_t N, int64_t K, const uint16_t *A,
                  int64_t lda, const uint16_t *B, int64_t ldb, float *C, int64_t ldc, void *workspace,
                  int64_t workspace_bytes, void *stream)
{
    int rc = check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc);
    if (rc != FSRGEMM_OK) return rc;
    if (!forced_ok(tile, kBf16_MainMore + kBf16MainShapes - 1, k_slices, M, N, K, 64, workspace, workspace_bytes)) return FSRGEMM_ERR_INVALID_ARG;
    const int a_lay = transA ? kMnContig : kKContig, b_lay = transB ? kKContig : kMnContig;
    Plan p = {tile, 0, k_slices};
    if (tile == kBf16_Vector) {
        if (M == 0 || N == 0) return FSRGEMM_OK;
        if (!vector_call_bf16(transA, transB, M, N, K, A, lda, B, ldb) || ceil_div(M > N ? M : N, 4) * k_slices >= ((int64_t)1 << 31)) return FSRGEMM_ERR_INVALID_ARG;
        return run_bf16(p, a_lay, b_lay, M, N, K, A, lda, B, ldb, C, ldc, static_cast<float *>(workspace), static_cast<hipStream_t>(stream));
    }
    rc = mode_bf16(tile, k_slices, M, N, K, A, lda, B, ldb, &p.mode);
    if (rc != FSRGEMM_OK) return rc;
    // a forced direct-to-LDS kernel is an invalid candidate where it does not fit; nothing else is substituted
    if (bf16_main_shape(tile) >= 0 && M > 0 && N > 0 &&
        (!bf16_main_fits(bf16_main_shape(tile), a_lay, b_lay, M, N, K, A, lda, B, ldb) || !bf16_main_slices_fit(K, k_slices)))
        return FSRGEMM_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return FSRGEMM_OK;
    return run_bf16(p, a_lay, b_lay, M, N, K, A, lda, B, ldb, C, ldc, static_cast<float *>(workspace),
                    static_cast<hipStream_t>(stream));
}

int fsrgemm_plan_bf16(int transA, int transB, int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda,
                      const uint16_t *B, int64_t ldb, int flags, int *tile, int *k_slices)
{
    if (!extents_ok(M, N, K) || tile == nullptr || k_slices == nullptr || (flags & ~3)) return FSRGEMM_ERR_INVALID_ARG;
    Plan p;
    const int rc = plan_bf16(transA ? kMnContig : kKContig, transB ? kKContig : kMnContig, M, N, K, A, lda, B, ldb,
                             (flags & 1) != 0, &p, (flags & 2) == 0);
    if (rc != FSRGEMM_OK) return rc;
    *tile = p.cfg;
    *k_slices = p.slices;
    return FSRGEMM_OK;
}

int fsrgemm_tile_count_bf16(void) { return kBf16_MainMore + kBf16MainShapes - 1; }

int fsrgemm_bands_bf16(int transA, int transB, int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda,
                       const uint16_t *B, int64_t ldb, int flags, int *dim, int64_t *at, int *tile_first, int *tile_second)
{
    if (!extents_ok(M, N, K) || dim == nullptr || at == nullptr || tile_first == nullptr || tile_second == nullptr || (flags & ~3)) return FSRGEMM_ERR_INVALID_ARG;
    Plan p;
    const int rc = plan_bf16(transA ? kMnContig : kKContig, transB ? kKContig : kMnContig, M, N, K, A, lda, B, ldb,
                             (flags & 1) != 0, &p, (flags & 2) == 0);
    if (rc != FSRGEMM_OK) return rc;
    *dim = p.band_dim, *at = p.band_at, *tile_first = p.cfg, *tile_second = p.band_dim ? p.cfg2 : p.cfg;
    return FSRGEMM_OK;
}

const char *fsrgemm_kernel_for_f32(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                                   int64_t ldb, const float *C, int64_t ldc)
{
    return fsrgemm_kernel_for_f32_ex(0, 0, M, N, K, A, lda, B, ldb, C, ldc);
}

const char *fsrgemm_kernel_for_f32_ex(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A,
                                      int64_t lda, const float *B, int64_t ldb, const float *C, int64_t ldc)
{
    Plan p;
    if (check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc) != FSRGEMM_OK) return nullptr;
    if (plan_f32(transA, transB, M, N, K, A, lda, B, ldb, false, &p) != FSRGEMM_OK) return nullptr;
    if (p.cfg >= kF32_Main) {
        const int a_lay = transA ? kMnContig : kKContig, b_lay = transB ? kKContig : kMnContig;
        const char *first = f32_main_kernel_name(p.cfg - kF32_Main, a_lay, b_lay);
        return p.band_dim == 0 ? first : two_band_name(p, first, f32_main_kernel_name(p.cfg2 - kF32_Main, a_lay, b_lay));
    }
    if (p.cfg == kF32_Vector) {
        const VecMap v = vector_map(transA, transB, M, N, K, A, lda, B, ldb, nullptr, ldc);
        return gemv_kernel_name(v.pattern, gemv_takes_vectors(v.a), v.a.nvec);
    }
    return f32_kernel_name(p.cfg, p.mode, transA ? kMnContig : kKContig, transB ? kKContig : kMnContig);
}

const char *fsrgemm_kernel_for_bf16(int64_t M, int64_t N, int64_t K, const uint16_t *A, int64_t lda,
                                    const uint16_t *B, int64_t ldb, const float *C, int64_t ldc)
{
    return fsrgemm_kernel_for_bf16_ex(0, 1, M, N, K, A, lda, B, ldb, C, ldc);
}

const char *fsrgemm_kernel_for_bf16_ex(int transA, int transB, int64_t M, int64_t N, int64_t K, const uint16_t *A,
                                       int64_t lda, const uint16_t *B, int64_t ldb, const float *C, int64_t ldc)
{
    Plan p;
    if (check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc) != FSRGEMM_OK) return nullptr;
    const int a_lay = transA ? kMnContig : kKContig, b_lay = transB ? kKContig : kMnContig;
    if (plan_bf16(a_lay, b_lay, M, N, K, A, lda, B, ldb, false, &p) != FSRGEMM_OK) return nullptr;
    if (p.cfg == kBf16_Vector) {
        const VecMap16 v = vector_map16(transA, transB, M, N, K, A, lda, B, ldb, nullptr, ldc);
        return gemv_bf16_kernel_name(v.pattern, gemv_bf16_takes_vectors(v.a), v.a.nvec, gemv_bf16_takes_mfma(v.pattern, v.a));
    }
    const char *first = bf16_kernel_name(p.cfg, p.mode, a_lay, b_lay);
    return p.band_dim == 0 ? first : two_band_name(p, first, bf16_kernel_name(p.cfg2, 0, a_lay, b_lay));
}

const char *fsrgemm_kernel_for_f32_cfg(int tile, int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A,
                                       int64_t lda, const float *B, int64_t ldb, const float *C, int64_t ldc)
{
    if (check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc) != FSRGEMM_OK) return nullptr;
    if (tile == kF32_Skinny) {
        // no kernel where no piece count gemm_f32_cfg accepts keeps the lane offsets of a piece in range
        SkinnyArgs sk;
        if (K < 1 || !tall_storage(transA, transB, M, N, lda, ldb, &sk.lda, &sk.ldb)) return nullptr;
        sk.K = (int)K, sk.parts = (int)(K < kSkinnyMaxParts ? K : kSkinnyMaxParts);
        if (!skinny_offsets_fit(sk)) return nullptr;
        return skinny_kernel_name((int)(M < 17 ? M : 17), (int)(N < 17 ? N : 17), A, sk.lda, B, sk.ldb);
    }
    if (tile >= kF32_Main && tile < kF32_Main + kF32MainShapes) {
        const int a_lay = transA ? kMnContig : kKContig, b_lay = transB ? kKContig : kMnContig;
        return f32_main_fits(tile - kF32_Main, a_lay, b_lay, M, N, K, A, lda, B, ldb) ? f32_main_kernel_name(tile - kF32_Main, a_lay, b_lay) : nullptr;
    }
    if (tile < 0 || tile > kF32_Vector || (tile == kF32_Vector && !vector_call_f32(transA, transB, M, N, K, A, lda, B, ldb))) return nullptr;
    int mode;
    if (mode_f32(tile, 1, M, N, K, A, lda, B, ldb, &mode) != FSRGEMM_OK) return nullptr;
    if (tile == kF32_Vector) {
        const VecMap v = vector_map(transA, transB, M, N, K, A, lda, B, ldb, nullptr, ldc);
        return gemv_kernel_name(v.pattern, gemv_takes_vectors(v.a), v.a.nvec);
    }
    return f32_kernel_name(tile, mode, transA ? kMnContig : kKContig, transB ? kKContig : kMnContig);
}

const char *fsrgemm_kernel_for_bf16_cfg(int tile, int transA, int transB, int64_t M, int64_t N, int64_t K,
                                        const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, const float *C,
                                        int64_t ldc)
{
    if (check_args(M, N, K, A, lda, transA ? M : K, B, ldb, transB ? K : N, C, ldc) != FSRGEMM_OK) return nullptr;
    if (tile == kBf16_Vector) {
        if (!vector_call_bf16(transA, transB, M, N, K, A, lda, B, ldb)) return nullptr;
        const VecMap16 v = vector_map16(transA, transB, M, N, K, A, lda, B, ldb, nullptr, ldc);
        return gemv_bf16_kernel_name(v.pattern, gemv_bf16_takes_vectors(v.a), v.a.nvec, gemv_bf16_takes_mfma(v.pattern, v.a));
    }
    if (tile < 0 || tile >= kBf16_MainMore + kBf16MainShapes - 1) return nullptr;
    const int a_lay = transA ? kMnContig : kKContig, b_lay = transB ? kKContig : kMnContig;
    int mode;
    if (mode_bf16(tile, 1, M, N, K, A, lda, B, ldb, &mode) != FSRGEMM_OK) return nullptr;
    if (bf16_main_shape(tile) >= 0 && !bf16_main_fits(bf16_main_shape(tile), a_lay, b_lay, M, N, K, A, lda, B, ldb)) return nullptr;
    return bf16_kernel_name(tile, mode, a_lay, b_lay);
}

static bool transpose_args_ok(int64_t rows, int64_t cols, const float *A, int64_t lda, const float *T, int64_t ldt)
{
    const int64_t lim = (int64_t)1 << 31;
    if (rows < 0 || cols < 0 || rows >= lim || cols >= lim || lda < cols || ldt < rows) return false;
    if (rows == 0 || cols == 0) return true;
    return A != nullptr && T != nullptr && ceil_div(rows, 64) * ceil_div(cols, 64) < lim;
}

const char *fsrgemm_kernel_for_transpose_f32(int64_t rows, int64_t cols, const float *A, int64_t lda, const float *T, int64_t ldt)
{
    if (!transpose_args_ok(rows, cols, A, lda, T, ldt)) return nullptr;
    return rows == 0 || cols == 0 ? "none" : transpose_kernel_name((int)rows, (int)cols);
}

int transpose_f32(int64_t rows, int64_t cols, const float *A, int64_t lda, float *T, int64_t ldt, void *stream)
{
    if (!transpose_args_ok(rows, cols, A, lda, T, ldt)) return FSRGEMM_ERR_INVALID_ARG;
    if (rows == 0 || cols == 0) return FSRGEMM_OK;
    const int rc = device_ok();
    if (rc != FSRGEMM_OK) return rc;
    const hipError_t e = launch_transpose_f32(A, lda, T, ldt, (int)rows, (int)cols, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FSRGEMM_OK : FSRGEMM_ERR_LAUNCH;
}

int fsrgemm_mfma_ceiling(int kind, int passes, const void *operands, float *sink, int workgroups, double *flop, void *stream)
{
    if (kind < 0 || kind > 1 || passes < 1 || passes > (1 << 24) || workgroups < 1 || workgroups > (1 << 16)) return FSRGEMM_ERR_INVALID_ARG;
    if (operands == nullptr || sink == nullptr || !aligned16(operands)) return FSRGEMM_ERR_INVALID_ARG;
    if (flop != nullptr) *flop = mfma_ceiling_flop(kind, passes, workgroups);
    const int rc = device_ok();
    if (rc != FSRGEMM_OK) return rc;
    return launch_mfma_ceiling(kind, passes, operands, sink, workgroups, static_cast<hipStream_t>(stream)) == hipSuccess ? FSRGEMM_OK : FSRGEMM_ERR_LAUNCH;
}

const char *fsrgemm_kernel_for_mfma_ceiling(int kind) { return kind == 0 || kind == 1 ? mfma_ceiling_kernel_name(kind) : nullptr; }

const char *fsrgemm_status_string(int status)
{
    switch (status) {
    case FSRGEMM_OK: return "ok";
    case FSRGEMM_ERR_INVALID_ARG: return "invalid argument";
    case FSRGEMM_ERR_LAUNCH: return "kernel launch failed";
    case FSRGEMM_ERR_UNSUPPORTED_DEVICE: return "current device is not gfx950";
    case FSRGEMM_ERR_SCRATCH_LIMIT: return "the problem's K split needs more scratch memory than the library's fixed buffer holds";
    default: return "unknown status";
    }
}

int fsrgemm_version(void) { return 300; }

}  // extern "C"
