/*
 * CPU oracle for matrix transposition (the paper's Task 8 in its task-prompt
 * table: a matrix of 32-bit floating point numbers with `rows` rows and
 * `cols` columns becomes one with `cols` rows and `rows` columns).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the GPU library includes, links or
 * calls this file; it shares no header, helper or constant with it.
 *
 * The definition is written out directly, one element at a time:
 *
 *     T[j][i] = A[i][j]        0 <= i < rows, 0 <= j < cols
 *
 * Elements are moved as 32-bit words, so every bit pattern (negative zero,
 * NaN payloads) arrives unchanged.  Both matrices are addressed through
 * explicit (row stride, column stride) pairs in elements, so row-major,
 * column-major and padded storage go through the same loop.
 */
#include <stdint.h>

int oracle_transpose_f32(int64_t rows, int64_t cols,
                         const uint32_t *A, int64_t a_rs, int64_t a_cs,
                         uint32_t *T, int64_t t_rs, int64_t t_cs)
{
    if (rows < 0 || cols < 0) return -1;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j)
            T[j * t_rs + i * t_cs] = A[i * a_rs + j * a_cs];
    return 0;
}
