/*
 * TEST INFRASTRUCTURE ONLY: slow, plain CPU definition of the storage change behind "running a
 * matrix multiply in another mode" (paper Sec. IV-C: the same product can be computed as NN, NT or
 * TN, which differ only in how each operand is laid out in memory).  Imported by tests/, the smoke
 * check and the benchmark's CPU leg; never by the product path.
 *
 * dst[c * rows + r] = src[r * cols + c] for 16-bit elements (bf16 bit patterns are moved, never
 * interpreted).  Returns 0, or -1 on a negative size or a null pointer with a non-empty matrix.
 */
#include <stddef.h>
#include <stdint.h>

int oracle_transpose_u16(int64_t rows, int64_t cols, const uint16_t *src, uint16_t *dst)
{
    if (rows < 0 || cols < 0) return -1;
    if (rows == 0 || cols == 0) return 0;
    if (!src || !dst) return -1;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c)
            dst[(size_t)c * (size_t)rows + (size_t)r] = src[(size_t)r * (size_t)cols + (size_t)c];
    return 0;
}
