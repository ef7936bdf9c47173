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
 *
 * Dense blocks with an error bound (same section: in dense blocks each element is predicted
 * from its neighbours by the Lorenzo predictor, prediction errors within the bound are
 * quantised, outliers are preserved intact, and prediction works on decompressed rather than
 * original values).  With eps > 0 a dense block is stored like this instead (eps <= 0 or NaN
 * keeps the verbatim form above; the paper's equations for this step are garbled and give
 * neither the bound, the predictor's order nor a code width):
 *
 *   lattice   two_eps = eps + eps; t = x / two_eps (binary32 division); an element is
 *             representable iff |t| < 2^22, and then q = (int)rintf(t); otherwise q = 0.
 *             The decompressed value of a representable element is (float)q * two_eps, which
 *             is within eps of x (up to the two roundings); predicting from these integers is
 *             predicting from decompressed values.
 *   predict   first-order Lorenzo in two dimensions, inside the block:
 *             p(r,c) = q(r,c-1) + q(r-1,c) - q(r-1,c-1), neighbours outside the block are 0.
 *   code      d = q - p; if the element is representable and -128 < d < 128 its code byte is
 *             d + 128 (1..255); otherwise the element is an outlier: code byte 0 and its
 *             original bits are appended to the value stream.
 *   info      0x80 | number of outliers (0..64); the value stream gets the outliers in
 *             row-major order, the index stream gets the block's area code bytes, row-major.
 *             (The verbatim form is the case "every element an outlier, no code bytes".)
 *   restore   row-major: a code byte 0 takes the next outlier, returns it unchanged and
 *             re-derives its q as above; any other code gives q = p + code - 128 and returns
 *             (float)q * two_eps (rounded to bf16, nearest even, for bf16 maps).
 *   Huffman coding of the code bytes, which the paper applies last, is a separate step on the
 *   index stream (fho_huffman.c).
 */
#include "fho.h"

#include <math.h>
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


/* ---- the error-bounded predictive form of dense blocks ---- */
static float bits_to_float(uint32_t bits, int dtype)
{
    uint32_t u = dtype == FHO_F32 ? bits : bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static uint32_t float_to_bits(float f, int dtype)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if (dtype == FHO_F32) return u;
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;             /* nearest even */
}

/* the lattice point of x; *ok = 0 when x has none (then the point is 0) */
static int32_t lattice(float x, float two_eps, int *ok)
{
    float t = x / two_eps;
    *ok = fabsf(t) < 0x1p22f;                                  /* false for NaN and infinities too */
    return *ok ? (int32_t)rintf(t) : 0;
}

static int predictive(float eps) { return eps > 0.0f; }

/* Encode one dense block; returns its number of outliers.  codes gets rows*cols bytes,
 * outliers (if not NULL) the original bits of the outliers. */
static int lorenzo_encode_block(const void *x, int dtype, int64_t origin, int64_t w, int rows, int cols,
                                float two_eps, uint8_t *codes, uint32_t *outliers)
{
    int32_t q[8][8];
    int nout = 0;
    for (int r = 0; r < rows; ++r) {
        for (int c = 0; c < cols; ++c) {
            uint32_t bits = elem_bits(x, dtype, origin + r * w + c);
            int ok;
            q[r][c] = lattice(bits_to_float(bits, dtype), two_eps, &ok);
            int32_t left = c > 0 ? q[r][c - 1] : 0, up = r > 0 ? q[r - 1][c] : 0;
            int32_t diag = (r > 0 && c > 0) ? q[r - 1][c - 1] : 0;
            int32_t d = q[r][c] - (left + up - diag);
            if (ok && d > -128 && d < 128) {
                codes[r * cols + c] = (uint8_t)(d + 128);
            } else {
                codes[r * cols + c] = 0;
                if (outliers) outliers[nout] = bits;
                ++nout;
            }
        }
    }
    return nout;
}

int fho_sparse_encode(const void *x, int dtype, int64_t maps, int64_t h, int64_t w, int n, float tau, float eps,
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
                } else if (predictive(eps)) {                  /* dense, within the error bound */
                    uint32_t out_bits[64];
                    int nout = lorenzo_encode_block(x, dtype, (m * h + r0) * w + c0, w, rows, cols, eps + eps,
                                                    indices + ni, out_bits);
                    for (int k = 0; k < nout; ++k) put_bits(values, dtype, (int64_t)nv + k, out_bits[k]);
                    info[b] = (uint8_t)(0x80 | nout);
                    nv += (uint64_t)nout;
                    ni += (uint64_t)area;
                    totals[3] += 1;
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
                      int64_t maps, int64_t h, int64_t w, int n, float eps, void *out)
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
                if ((info[b] & 0x80) && predictive(eps)) {
                    const float two_eps = eps + eps;
                    const uint8_t *codes = indices + ni;
                    int32_t q[8][8];
                    int used = 0;
                    for (int r = 0; r < rows; ++r) {
                        for (int c = 0; c < cols; ++c) {
                            int32_t left = c > 0 ? q[r][c - 1] : 0, up = r > 0 ? q[r - 1][c] : 0;
                            int32_t diag = (r > 0 && c > 0) ? q[r - 1][c - 1] : 0;
                            uint32_t bits;
                            if (codes[r * cols + c] == 0) {
                                if (used >= count) return -2;
                                bits = elem_bits(values, dtype, (int64_t)nv + used++);
                                int ok;
                                q[r][c] = lattice(bits_to_float(bits, dtype), two_eps, &ok);
                            } else {
                                q[r][c] = left + up - diag + ((int32_t)codes[r * cols + c] - 128);
                                bits = float_to_bits((float)q[r][c] * two_eps, dtype);
                            }
                            put_bits(out, dtype, (m * h + r0 + r) * w + c0 + c, bits);
                        }
                    }
                    if (used != count) return -2;
                    nv += (uint64_t)count;
                    ni += (uint64_t)(rows * cols);
                } else if (info[b] & 0x80) {
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
