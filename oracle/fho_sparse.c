/*
 * fho_sparse.c -- CPU oracle for the sparse-block storage of salient-channel feature maps
 * (paper Section 4.4.1: the non-zero values of an h x w channel map are split into dense
 * and sparse blocks, starting from a binary non-zero mask that is mean-filtered by average
 * pooling with an n x n window and compared with a sparsity threshold tau; sparse blocks are
 * stored in Compressed Sparse Row format; zeros must come back exactly).
 *
 * THIS IS TEST INFRASTRUCTURE (see fho.h).  Plain scalar C, host pointers.
 *
 * The paper gives the steps but not n, tau, the stride of the pooling or a storage layout.
 * The definition implemented here:
 *
 *   input     `maps` feature maps of h x w elements, row-major, contiguous ([maps][h][w]).
 *   blocks    the pooling is non-overlapping (stride n): map m is cut into
 *             BH x BW = ceil(h/n) x ceil(w/n) blocks; block (bi, bj) covers rows
 *             bi*n .. min(h, bi*n+n)-1 and columns bj*n .. min(w, bj*n+n)-1, so edge
 *             blocks are smaller; area = rows * cols of the block.  n is 2, 4 or 8.
 *             Blocks are numbered b = (m*BH + bi)*BW + bj.
 *   mask      an element is non-zero iff its bit pattern is not all zero (-0.0 therefore
 *             counts as a value and survives the round trip bit for bit).
 *   density   the average of the mask over the block's existing elements (average pooling
 *             that does not count padding): density = (float)nnz / (float)area, one
 *             binary32 division.
 *   split     the block is sparse iff density <= tau (binary32 compare), else dense.
 *   info      one byte per block: bit 7 = dense, bits 0..6 = count, where count = nnz for a
 *             sparse block and area for a dense one (both <= 64).
 *   values    one stream of elements in block order: a sparse block contributes its nnz
 *             non-zero values in row-major order, a dense block all its area values in
 *             row-major order.
 *   indices   one byte stream in block order; a sparse block contributes its CSR structure:
 *             row_ptr[0..rows] (row_ptr[r] = non-zeros in the block's rows before r) followed
 *             by the column (0..cols-1, inside the block) of each non-zero in row-major
 *             order; a dense block contributes nothing.
 *   totals    {values written, index bytes written, sparse blocks, dense blocks}.
 *   restore   blocks are walked in order with running offsets into the two streams: a
 *             sparse block is zero-filled (+0.0) and its values scattered through the CSR
 *             structure, a dense block is copied.  The round trip is lossless.
 */
#include "fho.h"

#include <string.h>

static int sparse_args_ok(int64_t maps, int64_t h, int64_t w, int n, int dtype)
{
    if (maps < 0 || h < 1 || w < 1) return 0;
    if (n != 2 && n != 4 && n != 8) return 0;
    if (dtype != FHO_F32 && dtype != FHO_BF16) return 0;
    return 1;
}

int64_t fho_sparse_blocks(int64_t maps, int64_t h, int64_t w, int n)
{
    if (maps < 0 || h < 1 || w < 1 || n < 1) return -1;
    return maps * ((h + n - 1) / n) * ((w + n - 1) / n);
}

/* bit pattern of element i, widened to 32 bits */
static uint32_t elem_bits(const void *x, int dtype, int64_t i)
{
    return dtype == FHO_F32 ? ((const uint32_t *)x)[i] : (uint32_t)((const uint16_t *)x)[i];
}

static void put_bits(void *dst, int dtype, int64_t i, uint32_t bits)
{
    if (dtype == FHO_F32) ((uint32_t *)dst)[i] = bits;
    else ((uint16_t *)dst)[i] = (uint16_t)bits;
}

int fho_sparse_encode(const void *x, int dtype, int64_t maps, int64_t h, int64_t w, int n, float tau,
                      uint8_t *info, void *values, uint8_t *indices, uint64_t totals[4])
{
    if (!sparse_args_ok(maps, h, w, n, dtype) || !totals) return -1;
    totals[0] = totals[1] = totals[2] = totals[3] = 0;
    if (maps == 0) return 0;
    if (!x || !info || !values || !indices) return -1;
    const int64_t BH = (h + n - 1) / n, BW = (w + n - 1) / n;
    uint64_t nv = 0, ni = 0;
    int64_t b = 0;
    for (int64_t m = 0; m < maps; ++m) {
        for (int64_t bi = 0; bi < BH; ++bi) {
            for (int64_t bj = 0; bj < BW; ++bj, ++b) {
                const int64_t r0 = bi * n, c0 = bj * n;
                const int rows = (int)(h - r0 < n ? h - r0 : n), cols = (int)(w - c0 < n ? w - c0 : n);
                const int area = rows * cols;
                int nnz = 0;
                for (int r = 0; r < rows; ++r)
                    for (int c = 0; c < cols; ++c)
                        if (elem_bits(x, dtype, (m * h + r0 + r) * w + c0 + c) != 0u) ++nnz;
                const float density = (float)nnz / (float)area;
                if (density <= tau) {                          /* sparse: CSR */
                    info[b] = (uint8_t)nnz;
                    uint8_t *row_ptr = indices + ni;
                    uint8_t *col = row_ptr + rows + 1;
                    int k = 0;
                    for (int r = 0; r < rows; ++r) {
                        row_ptr[r] = (uint8_t)k;
                        for (int c = 0; c < cols; ++c) {
                            uint32_t bits = elem_bits(x, dtype, (m * h + r0 + r) * w + c0 + c);
                            if (bits != 0u) {
                                put_bits(values, dtype, (int64_t)nv + k, bits);
                                col[k] = (uint8_t)c;
                                ++k;
                            }
                        }
                    }
                    row_ptr[rows] = (uint8_t)k;
                    nv += (uint64_t)nnz;
                    ni += (uint64_t)(rows + 1 + nnz);
                    totals[2] += 1;
                } else {                                       /* dense: verbatim */
                    info[b] = (uint8_t)(0x80 | area);
                    int k = 0;
                    for (int r = 0; r < rows; ++r)
                        for (int c = 0; c < cols; ++c, ++k)
                            put_bits(values, dtype, (int64_t)nv + k, elem_bits(x, dtype, (m * h + r0 + r) * w + c0 + c));
                    nv += (uint64_t)area;
                    totals[3] += 1;
                }
            }
        }
    }
    totals[0] = nv;
    totals[1] = ni;
    return 0;
}

int fho_sparse_decode(const uint8_t *info, const void *values, const uint8_t *indices, int dtype,
                      int64_t maps, int64_t h, int64_t w, int n, void *out)
{
    if (!sparse_args_ok(maps, h, w, n, dtype)) return -1;
    if (maps == 0) return 0;
    if (!info || !values || !indices || !out) return -1;
    const int64_t BH = (h + n - 1) / n, BW = (w + n - 1) / n;
    uint64_t nv = 0, ni = 0;
    int64_t b = 0;
    for (int64_t m = 0; m < maps; ++m) {
        for (int64_t bi = 0; bi < BH; ++bi) {
            for (int64_t bj = 0; bj < BW; ++bj, ++b) {
                const int64_t r0 = bi * n, c0 = bj * n;
                const int rows = (int)(h - r0 < n ? h - r0 : n), cols = (int)(w - c0 < n ? w - c0 : n);
                const int count = info[b] & 0x7f;
                if (info[b] & 0x80) {
                    if (count != rows * cols) return -2;       /* not a stream this encoder wrote */
                    int k = 0;
                    for (int r = 0; r < rows; ++r)
                        for (int c = 0; c < cols; ++c, ++k)
                            put_bits(out, dtype, (m * h + r0 + r) * w + c0 + c, elem_bits(values, dtype, (int64_t)nv + k));
                    nv += (uint64_t)count;
                } else {
                    const uint8_t *row_ptr = indices + ni;
                    const uint8_t *col = row_ptr + rows + 1;
                    if (row_ptr[0] != 0 || row_ptr[rows] != count) return -2;
                    for (int r = 0; r < rows; ++r) {
                        for (int c = 0; c < cols; ++c) put_bits(out, dtype, (m * h + r0 + r) * w + c0 + c, 0u);
                        for (int k = row_ptr[r]; k < row_ptr[r + 1]; ++k) {
                            if (col[k] >= cols) return -2;
                            put_bits(out, dtype, (m * h + r0 + r) * w + c0 + col[k], elem_bits(values, dtype, (int64_t)nv + k));
                        }
                    }
                    nv += (uint64_t)count;
                    ni += (uint64_t)(rows + 1 + count);
                }
            }
        }
    }
    return 0;
}
