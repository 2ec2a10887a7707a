/*
 * fsrgemm -- dense matrix multiplication C = A x B for AMD MI355X (gfx950)
 * (and, at the end of this file, matrix transposition).
 *
 * The operation is the one the paper states for its Task 2 (task-prompt
 * table in the appendix): given A of M x K and B of K x N, produce the
 * M x N product.  There is no alpha/beta scaling and C is overwritten.
 * The paper's Function Validator and Performance Profiler (Section 3.2)
 * call a kernel through a fixed host harness that owns all memory; this
 * library plays the kernel's part and leaves allocation, transfers and
 * result checking to the caller in the same way.
 *
 * Conventions shared by every entry point
 *   - All matrix pointers are DEVICE pointers, valid on the current HIP
 *     device.  The library allocates nothing and keeps no workspace
 *     (the *_ws entry points take one from the caller).
 *   - M, N, K and the leading dimensions are counted in ELEMENTS.
 *   - Pointers need only the natural alignment of their element type;
 *     the fastest kernels are picked automatically when base addresses
 *     and leading dimensions are multiples of 16 bytes.  M and N may be
 *     any size; K is fastest as a multiple of 16 (fp32) or 64 (bf16).
 *   - A, B and C must not overlap.  Padding (columns N..ldc-1 of C) is
 *     never written; padding of A and B is never read.
 *   - M == 0 or N == 0: nothing is launched, FSRGEMM_OK.  K == 0: the
 *     M x N block of C is set to +0 (empty sum).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default
 *     stream).  The call enqueues work and returns without synchronising.
 *   - Results are deterministic: the same inputs give bit-identical C.
 *   - Entry points may be called from several host threads at once.
 *   - Errors are reported through the return value only.  Argument errors
 *     are detected before any HIP call is made, so they can be exercised on
 *     a machine without a GPU.
 */
#ifndef FSRGEMM_H
#define FSRGEMM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FSRGEMM_OK = 0,
    /* negative extent, leading dimension too small, NULL pointer with a
     * non-empty matrix, or an extent beyond the supported range */
    FSRGEMM_ERR_INVALID_ARG = -1,
    /* the HIP runtime refused the launch (kept apart from a wrong result,
     * as the paper's refinement prompts keep "failed to launch" apart from
     * "output mismatch", Appendix B) */
    FSRGEMM_ERR_LAUNCH = -2,
    /* current device is not gfx950 */
    FSRGEMM_ERR_UNSUPPORTED_DEVICE = -3,
    /* gemm_f32_noalloc only: the K split planned for the problem needs more
     * scratch memory than the library's fixed buffer holds */
    FSRGEMM_ERR_SCRATCH_LIMIT = -4
} fsrgemm_status;

/*
 * fp32 product, the precision of the paper's Task 2.
 *   C[M x N] = A[M x K] . B[K x N], all three ROW-major:
 *   A[i][k] at A[i*lda + k] (lda >= K), B[k][j] at B[k*ldb + j] (ldb >= N),
 *   C[i][j] at C[i*ldc + j] (ldc >= N).
 * Products and sums are IEEE fp32 (matrix-core FMA chains, no reduced
 * precision); the order of summation over k is fixed but unspecified.
 * M, N, K must each be < 2^31.
 */
int gemm_f32(int64_t M, int64_t N, int64_t K,
             const float *A, int64_t lda,
             const float *B, int64_t ldb,
             float *C, int64_t ldc,
             void *stream);

/*
 * The same fp32 product with either operand stored transposed.  The paper's task table defines Task 2 by
 * its shapes only and names a storage order (row-major) just for its convolution and transpose tasks, so a
 * harness may hold either operand either way.
 *   transA == 0: A[i][k] at A[i*lda + k] (lda >= K);  transA != 0: A[i][k] at A[k*lda + i] (lda >= M)
 *   transB == 0: B[k][j] at B[k*ldb + j] (ldb >= N);  transB != 0: B[k][j] at B[j*ldb + k] (ldb >= K)
 * C is row-major as in gemm_f32, and gemm_f32(...) is gemm_f32_ex(0, 0, ...).  Everything else
 * (arithmetic, alignment rules, empty extents, errors) is as for gemm_f32.
 */
int gemm_f32_ex(int transA, int transB,
                int64_t M, int64_t N, int64_t K,
                const float *A, int64_t lda,
                const float *B, int64_t ldb,
                float *C, int64_t ldc,
                void *stream);

/*
 * fp32 product with a caller-provided device workspace.  The paper's validator runs a kernel on inputs of
 * several sizes (Section 3.2, appendix table of test sizes); for the sizes with few output elements and a long
 * K -- a row or column vector times a matrix, a small square of long dot products -- too few output tiles
 * exist to occupy the device.  With a workspace such problems are cut along K: every slice's partial product
 * goes to the workspace and a second kernel adds the slices in slice order, so the result is still the same
 * on every call (it may differ in the last bits from gemm_f32_ex, which sums along K in one piece).
 *   gemm_f32_workspace_bytes: bytes that make the split possible for this shape, 0 when the problem is not
 *     split (the answer depends on M, N, K and the storage orders only; at most 16 MiB).  How a problem is cut
 *     also depends on the operands' alignment (16-byte aligned bases and rows let the direct-to-LDS kernel take
 *     the slices); the figure is the larger of the two needs, so a call may use less of the workspace than it names.
 *   gemm_f32_ws: as gemm_f32_ex; `workspace` is device memory of `workspace_bytes` bytes, 4-byte aligned, not
 *     overlapping A, B or C, owned by the caller and free for reuse once the stream has passed the call.
 *     Its contents on entry are ignored, on exit unspecified.  With a NULL, misaligned or too small workspace
 *     the call does exactly what gemm_f32_ex does.  Calls that share one workspace must be ordered by the
 *     caller (same stream, or events).
 */
int64_t gemm_f32_workspace_bytes(int transA, int transB, int64_t M, int64_t N, int64_t K);
int gemm_f32_ws(int transA, int transB,
                int64_t M, int64_t N, int64_t K,
                const float *A, int64_t lda,
                const float *B, int64_t ldb,
                float *C, int64_t ldc,
                void *workspace, int64_t workspace_bytes,
                void *stream);

/*
 * gemm_f32_ws for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Arguments and result are gemm_f32_ws's with a workspace of the size
 * gemm_f32_workspace_bytes names (bit for bit the same C), but the workspace is a fixed array of
 * FSRGEMM_NOALLOC_SCRATCH_BYTES inside the library's device image: each GPU the library runs on holds its own
 * copy until the process ends.  The call allocates and frees nothing (no hipMalloc, hipFree or allocating library
 * routine); the array's address is looked up on the first call on each device.
 *   - The array is as large as the largest workspace gemm_f32_workspace_bytes ever names (16 MiB), so every problem
 *     gemm_f32_ws can split is split here in the same way.  Should a plan ever need more than the array holds, the
 *     call returns FSRGEMM_ERR_SCRATCH_LIMIT before anything is launched (gemm_f32_ex computes any problem unsplit).
 *     Problems that are not split (gemm_f32_workspace_bytes == 0) never touch the array.
 *   - Every call on one GPU shares that GPU's array, whatever its stream or host thread.  Nothing in it has to start
 *     at zero (every partial product is written before it is read), so calls need no clearing between them, but
 *     calls that overlap in time on one GPU race on it: order them (one stream, or events) as calls that share a
 *     workspace must be ordered.
 */
#define FSRGEMM_NOALLOC_SCRATCH_BYTES 16777216 /* 16 MiB */
int gemm_f32_noalloc(int transA, int transB,
                     int64_t M, int64_t N, int64_t K,
                     const float *A, int64_t lda,
                     const float *B, int64_t ldb,
                     float *C, int64_t ldc,
                     void *stream);

/*
 * bf16 inputs, fp32 accumulation and fp32 output.
 *   A is ROW-major bf16: A[i][k] at A[i*lda + k] (lda >= K).
 *   B is COLUMN-major bf16: B[k][j] at B[j*ldb + k] (ldb >= K), i.e. both
 *   operands are contiguous along k.
 *   C is row-major fp32 (ldc >= N).
 * bf16 values are raw 16-bit patterns (the upper half of an IEEE fp32
 * word).  Each product is exact in fp32; sums are fp32.
 */
int gemm_bf16(int64_t M, int64_t N, int64_t K,
              const uint16_t *A, int64_t lda,
              const uint16_t *B, int64_t ldb,
              float *C, int64_t ldc,
              void *stream);

/*
 * The bf16 product with either operand in either storage order; transA / transB mean what they mean for
 * gemm_f32_ex (transB == 0 is a ROW-major B, B[k][j] at B[k*ldb + j], ldb >= N), so
 * gemm_bf16(...) is gemm_bf16_ex(0, 1, ...).  Operands that are contiguous along m or n are regrouped on
 * their way into on-chip memory; the fastest path is the one gemm_bf16 takes.
 */
int gemm_bf16_ex(int transA, int transB,
                 int64_t M, int64_t N, int64_t K,
                 const uint16_t *A, int64_t lda,
                 const uint16_t *B, int64_t ldb,
                 float *C, int64_t ldc,
                 void *stream);

/*
 * The bf16 product with a caller-provided workspace: gemm_bf16_ex's arguments, gemm_f32_ws's workspace rules
 * (partial products are fp32; the split depends on M, N, K only; at most 16 MiB).
 */
int64_t gemm_bf16_workspace_bytes(int transA, int transB, int64_t M, int64_t N, int64_t K);
int gemm_bf16_ws(int transA, int transB,
                 int64_t M, int64_t N, int64_t K,
                 const uint16_t *A, int64_t lda,
                 const uint16_t *B, int64_t ldb,
                 float *C, int64_t ldc,
                 void *workspace, int64_t workspace_bytes,
                 void *stream);

/*
 * The products with the configuration chosen by the caller instead of the dispatcher: the candidates of a
 * selection loop shaped like the paper's Algorithm 1 (generate candidates, drop those that fail to build or to
 * validate, keep the one with the least measured time), with tile configurations and K slices in the place of
 * generated kernels.
 *   tile: fp32  0 = 256 x 128, 1 = 128 x 128, 2 = 64 x 64 output tile per workgroup, 3 = the streaming kernels for
 *               M == 1 or N == 1 with K > 0, which use no matrix cores, and for M <= 16 or N <= 16 (any alignment) unless
 *               the operand on the other side (B for M < N, else A) is stored contiguous along n (m) and N (M) < 4;
 *               4 = the kernel for small results of long
 *               sums (both operands stored with k as the row index: transA != 0 or M == 1, transB == 0 or N == 1; M, N <= 16 with
 *               at most 144 entries after rounding both up to multiples of 4; K > 0), whose
 *               k_slices are workgroups (1..256, at most K) that each keep a partial result in the workspace, so it
 *               needs its workspace even for one, 5..16 = the direct-to-LDS kernel with tiles 256 x 256, 192 x 256,
 *               128 x 256, 256 x 128, 192 x 128, 128 x 128, 256 x 192, 192 x 192, 128 x 192, 64 x 64, 128 x 64,
 *               64 x 128 (fsrgemm_tile_count_f32() = 17);
 *         bf16  0 = 256 x 256 with direct-to-LDS loads, 1 = 256 x 256, 2 = 128 x 128, 3 = 64 x 64, 4 = the streaming
 *               kernels for M == 1 or N == 1 with K > 0, and for M <= 8 or N <= 8 (any alignment) unless the operand on
 *               the other side (B for M < N, else A) is stored contiguous along n (m) and N (M) < 8; with transA == 0, transB != 0, K a multiple of 8 and both
 *               operands 16-byte aligned with leading dimensions that are multiples of 8 also for M <= 16 or N <= 16 (a
 *               streaming kernel on the matrix cores); 5..10 = the direct-to-LDS kernel with tiles 192 x 256,
 *               128 x 256, 256 x 192, 192 x 192, 256 x 128, 128 x 128 (fsrgemm_tile_count_bf16() = 11).
 *   k_slices: 1 = K in one piece; 2..64 = split along K as gemm_f32_ws does, which needs a workspace of
 *         k_slices * M * N * 4 bytes (4-byte aligned, at most 16 MiB) and k_slices <= ceil(K / 16) (fp32) or
 *         ceil(K / 64) (bf16).
 * A candidate that cannot run this problem is FSRGEMM_ERR_INVALID_ARG and launches nothing: a tile or slice
 * count out of range, a split without a fitting workspace, fp32 candidate 3 or bf16 candidate 4 on a product
 * without 1 .. 16 (bf16: 8, and 16 only where described above) rows or columns on one side,
 * fp32 candidate 4 on a result that is too large,
 * fp32 tiles 5..16 where their kernel's conditions fail (M, N at least one tile, K >= 32 and a
 * multiple of 4, 16-byte aligned operands with leading dimensions that are multiples of 4 and below 2^24;
 * M or N a multiple of 4 for an operand contiguous along it) or with a slice count that does not leave every
 * slice a whole K-tile (slices are ceil(ceil(K / 32) / k_slices) K-tiles of 32 long, the last one takes the rest),
 * bf16 tiles 0 and 5..10 where their kernel's
 * conditions fail (M, N at least one tile, K >= 64 and a multiple of 8, 16-byte aligned operands with leading
 * dimensions that are multiples of 8 and below 2^25; with an operand contiguous along m or n, M or N a multiple
 * of 8) or with a slice count that does not leave every slice a whole K-tile (slices are
 * ceil(ceil(K / 64) / k_slices) K-tiles of 64 long, the last one takes the rest).  Every other
 * candidate takes any shape and alignment.  All other arguments as for gemm_f32_ws / gemm_bf16_ws.
 */
int gemm_f32_cfg(int tile, int k_slices, int transA, int transB,
                 int64_t M, int64_t N, int64_t K,
                 const float *A, int64_t lda,
                 const float *B, int64_t ldb,
                 float *C, int64_t ldc,
                 void *workspace, int64_t workspace_bytes,
                 void *stream);
int gemm_bf16_cfg(int tile, int k_slices, int transA, int transB,
                  int64_t M, int64_t N, int64_t K,
                  const uint16_t *A, int64_t lda,
                  const uint16_t *B, int64_t ldb,
                  float *C, int64_t ldc,
                  void *workspace, int64_t workspace_bytes,
                  void *stream);
int fsrgemm_tile_count_f32(void);
int fsrgemm_tile_count_bf16(void);

/*
 * What the dispatcher would choose for this problem, in the terms of the *_cfg calls: the starting point of a
 * selection run.  flags: FSRGEMM_PLAN_WORKSPACE = the choice of a *_ws call whose workspace is big enough;
 * FSRGEMM_PLAN_RULES_ONLY = the choice of the built-in rules alone, without the library's table of earlier
 * selection results (which otherwise decides for a problem -- precision, storage orders, M, N, K -- that has a
 * row there).  A and B are looked at for their alignment only (no device access).  Returns FSRGEMM_OK and sets
 * *tile, *k_slices, or FSRGEMM_ERR_INVALID_ARG.  Where the product runs as two bands (below), *tile is the
 * first band's.
 */
#define FSRGEMM_PLAN_WORKSPACE 1
#define FSRGEMM_PLAN_RULES_ONLY 2
int fsrgemm_plan_f32(int transA, int transB, int64_t M, int64_t N, int64_t K,
                     const float *A, int64_t lda, const float *B, int64_t ldb,
                     int flags, int *tile, int *k_slices);
int fsrgemm_plan_bf16(int transA, int transB, int64_t M, int64_t N, int64_t K,
                      const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
                      int flags, int *tile, int *k_slices);

/*
 * Two bands.  A launch lasts as long as the compute unit with the most output tiles, so a problem whose tiles do
 * not fill whole rounds of the 256 compute units in any tile shape wastes part of its last round.  For such a
 * problem (large, aligned, not in the selection table, no K slices) the dispatcher may cut C once, along its rows or
 * its columns, and run each band as a product of its own, in the tile shape that suits that band's tile count:
 * two launches on the caller's stream, every entry of C still computed by one workgroup, the result the same bits
 * as in one launch (part of the tile configuration of Section 3.2's candidates: what is chosen, not what is computed).
 * These queries report that choice for the plain entry points (flags as for fsrgemm_plan_*):
 *   *dim          0: one launch; 1: rows [0, *at) and [*at, M); 2: columns [0, *at) and [*at, N)
 *   *at           the cut, a multiple of 64 (0 when *dim is 0)
 *   *tile_first, *tile_second   candidate numbers of the two bands' configurations (equal when *dim is 0)
 * A band of its own is exactly the forced call gemm_*_cfg(tile, 1, ...) on that band's rows or columns.
 * Returns FSRGEMM_OK or FSRGEMM_ERR_INVALID_ARG (NULL result pointers, extents out of range, unknown flags).
 */
int fsrgemm_bands_f32(int transA, int transB, int64_t M, int64_t N, int64_t K,
                      const float *A, int64_t lda, const float *B, int64_t ldb,
                      int flags, int *dim, int64_t *at, int *tile_first, int *tile_second);
int fsrgemm_bands_bf16(int transA, int transB, int64_t M, int64_t N, int64_t K,
                       const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
                       int flags, int *dim, int64_t *at, int *tile_first, int *tile_second);

/*
 * Name of the kernel variant the dispatcher would launch for this problem
 * (same argument checks as the gemm calls; launches nothing, touches no
 * device memory).  Returns a pointer to static storage, or NULL when the
 * arguments are invalid; for a product that runs as two bands the text is
 * "<first kernel> + <second kernel> (rows | columns from <cut>)" in a buffer
 * of the calling thread, valid until that thread's next such query.  The Performance-Profiler side of the bench uses it
 * to label timings and to find the kernel in a profiler trace.
 */
const char *fsrgemm_kernel_for_f32(int64_t M, int64_t N, int64_t K,
                                   const float *A, int64_t lda,
                                   const float *B, int64_t ldb,
                                   const float *C, int64_t ldc);
const char *fsrgemm_kernel_for_f32_ex(int transA, int transB,
                                      int64_t M, int64_t N, int64_t K,
                                      const float *A, int64_t lda,
                                      const float *B, int64_t ldb,
                                      const float *C, int64_t ldc);
const char *fsrgemm_kernel_for_bf16(int64_t M, int64_t N, int64_t K,
                                    const uint16_t *A, int64_t lda,
                                    const uint16_t *B, int64_t ldb,
                                    const float *C, int64_t ldc);

const char *fsrgemm_kernel_for_bf16_ex(int transA, int transB,
                                       int64_t M, int64_t N, int64_t K,
                                       const uint16_t *A, int64_t lda,
                                       const uint16_t *B, int64_t ldb,
                                       const float *C, int64_t ldc);

/* The kernel a *_cfg call with this tile would launch, or NULL where the call would reject the candidate. */
const char *fsrgemm_kernel_for_f32_cfg(int tile, int transA, int transB,
                                       int64_t M, int64_t N, int64_t K,
                                       const float *A, int64_t lda,
                                       const float *B, int64_t ldb,
                                       const float *C, int64_t ldc);
const char *fsrgemm_kernel_for_bf16_cfg(int tile, int transA, int transB,
                                        int64_t M, int64_t N, int64_t K,
                                        const uint16_t *A, int64_t lda,
                                        const uint16_t *B, int64_t ldb,
                                        const float *C, int64_t ldc);

/*
 * Matrix transposition, the paper's Task 8 (task-prompt table: a rows x cols matrix of 32-bit floating point
 * numbers becomes a cols x rows one, all matrices row-major), the memory-bound counterpart of the product:
 *   T[j][i] = A[i][j]:  A[i][j] at A[i*lda + j] (lda >= cols),  T[j][i] at T[j*ldt + i] (ldt >= rows).
 * Values are moved as 32-bit words, so every bit pattern arrives unchanged.  A and T must not overlap (the
 * operation is out of place); padding of T (columns rows..ldt-1) is never written.  rows == 0 or cols == 0:
 * nothing is launched.  Pointers need only 4-byte alignment.  Conventions otherwise as for the products.
 */
int transpose_f32(int64_t rows, int64_t cols,
                  const float *A, int64_t lda,
                  float *T, int64_t ldt,
                  void *stream);

/* Name of the kernel variant transpose_f32 would launch (rules as for the queries above; "none" for an empty matrix). */
const char *fsrgemm_kernel_for_transpose_f32(int64_t rows, int64_t cols,
                                             const float *A, int64_t lda,
                                             const float *T, int64_t ldt);

/* Human-readable text for a status code; static storage, never NULL. */
/*
 * Measurement aid for the Performance Profiler leg (Section 3.2: candidates are ranked by measured execution time;
 * this gives the time a scale): a loop of nothing but the matrix-core instruction of the product kernels, one
 * wavefront per SIMD with all 256 accumulator registers in use, operands held in registers.  What it sustains is
 * the ceiling of the contraction step on this part for operands of this kind; it depends on the operand VALUES
 * (the clock follows the power drawn), which is why the caller supplies them.
 *   kind        0: V_MFMA_F32_32X32X2_F32 (the fp32 kernels), 1: V_MFMA_F32_16X16X32_BF16 (the bf16 kernels), issued
 *               in the order the product kernels issue them (kind 1: the two k-steps of a block back to back)
 *   passes      1 .. 2^24 loop iterations of 64 (kind 0) or 128 (kind 1) MFMAs per wavefront
 *   operands    device pointer, 16-byte aligned, to 8 KB (kind 0: 2048 floats) or 32 KB (kind 1: 16384 bf16 bit
 *               patterns); read once per lane, any finite values
 *   sink        device pointer to workgroups * 256 floats, overwritten with sums nobody needs
 *   workgroups  1 .. 65536 workgroups of 256 lanes; one per compute unit (256 on MI355X) loads the whole chip once
 *   flop        if not NULL, receives the floating-point operations of the launch:
 *               workgroups * 4 * passes * (64 * 4096 for kind 0, 128 * 16384 for kind 1)
 * Errors: FSRGEMM_ERR_INVALID_ARG for anything outside these ranges or a NULL / misaligned pointer, before any HIP call.
 */
int fsrgemm_mfma_ceiling(int kind, int passes, const void *operands, float *sink, int workgroups, double *flop,
                         void *stream);
/* Name of that kernel as a profiler trace prints it; NULL for an unknown kind. */
const char *fsrgemm_kernel_for_mfma_ceiling(int kind);

const char *fsrgemm_status_string(int status);

/* Library version as major*10000 + minor*100 + patch. */
int fsrgemm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FSRGEMM_H */
