/*
 * CPU oracle for the Endor bitmap sparse format.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain, sequential statement of what the format's two
 * algorithms compute.  It exists so that the GPU library can be checked against
 * something written straight from the paper.  It shares no code, header, table
 * or helper with the GPU library, and nothing in the product path may call it:
 * only the tests, the smoke check and the benchmark's CPU-baseline leg do.
 *
 * What follows the paper, and where:
 *   - oracle_compress    : Algorithm 1 (compression), Section 4.1 "Compression".
 *   - oracle_decompress  : Algorithm 2 (decompression), Section 4.1 "Decompression".
 *   - the layout (one bit per element, stored as a 1-d vector, plus the packed
 *     non-zero values in row-major order) : Figure "Sparse format" and Section 4.1.
 *
 * Readings taken where the paper is silent or its listing is garbled:
 *   R1. The bitmap b is the concatenation of the per-row lists b_i of Alg. 1, so
 *       the bit of element (i, j) has flat index e = i*cols + j; v is the
 *       concatenation of the v_i, and the counter k of Alg. 2 keeps running from
 *       one row to the next (the listing's per-row reset of k describes filling
 *       one row out of that row's own list v_i).
 *   R2. Alg. 2 has no else branch; a position whose bit is 0 receives the
 *       all-zero bit pattern, so the whole output is defined.
 *   R3. Bit order: bit e lives in byte e>>3 at bit position e&7 (LSB first).
 *   R4. No per-row padding: the bit stream is continuous over rows*cols bits;
 *       only the last byte may hold pad bits, written as 0 and never read.
 *   R5. "W[i,j] != 0" is a test on the element's bit pattern (any pattern other
 *       than all-zero is kept), so -0.0, subnormals, Inf and NaN of an fp16
 *       matrix survive a round trip bit for bit.
 *   R6. Elements are opaque 1- or 2-byte patterns (fp16 is the paper's main
 *       case; the 1-byte case is the INT8 variant of Section 4.2).  No floating
 *       point instruction ever touches a value.
 *
 * Algorithms 1 and 2 and the tables derived from them are integer / byte work, so
 * their results are exact.  The floating-point routines at the end of the file
 * (oracle_gemv_f16, oracle_gemm_f16_rows: the products of the decompressed matrix with
 * one or a few vectors) convert fp16 to double exactly and accumulate in double.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>

static int elem_is_nonzero(const uint8_t *p, int elem_bytes)
{
    int nz = 0;
    for (int b = 0; b < elem_bytes; ++b) nz |= (p[b] != 0);
    return nz;
}

/* Number of bytes the bitmap of a rows x cols matrix occupies: ceil(rows*cols/8)
 * (Section 4.1's size example: 9216*36864/8 bytes, no padding). */
int64_t oracle_bitmap_bytes(int64_t rows, int64_t cols)
{
    return (rows * cols + 7) / 8;
}

/*
 * Algorithm 1.  Visit the rows in order and, inside a row, the columns in
 * order.  A non-zero element is appended to v and a 1 is appended to b; a zero
 * element appends a 0 to b.
 *
 * dense       rows*cols elements of elem_bytes bytes each, row-major, contiguous
 * bitmap      out, oracle_bitmap_bytes(rows, cols) bytes
 * values      out, room for every non-zero (at most rows*cols elements); may be
 *             NULL to only count
 * row_offsets out or NULL, rows+1 entries: row_offsets[i] = number of non-zeros
 *             in rows before i (the length of v_0 .. v_{i-1} concatenated)
 * returns     nnz, the length of v
 */
int64_t oracle_compress(const void *dense, int elem_bytes, int64_t rows, int64_t cols,
                        uint8_t *bitmap, void *values, int64_t *row_offsets)
{
    const uint8_t *W = (const uint8_t *)dense;
    uint8_t *v = (uint8_t *)values;
    int64_t k = 0;
    memset(bitmap, 0, (size_t)oracle_bitmap_bytes(rows, cols));
    for (int64_t i = 0; i < rows; ++i) {
        if (row_offsets) row_offsets[i] = k;
        for (int64_t j = 0; j < cols; ++j) {
            int64_t e = i * cols + j;
            const uint8_t *w = W + e * elem_bytes;
            if (elem_is_nonzero(w, elem_bytes)) {
                if (v) memcpy(v + k * elem_bytes, w, (size_t)elem_bytes);
                k += 1;
                bitmap[e >> 3] |= (uint8_t)(1u << (e & 7));
            }
        }
    }
    if (row_offsets) row_offsets[rows] = k;
    return k;
}

/*
 * Algorithm 2 over a block of rows [row_begin, row_end).  k starts at k_begin,
 * the number of non-zeros in the rows before row_begin (0 for the whole
 * matrix).  Walk the positions in row-major order; where the bit is 1 the next
 * unread element of v is placed, where it is 0 the element is all-zero bits.
 *
 * out         the FULL rows x cols output; only rows [row_begin,row_end) are written
 * returns     k after the last row (for the whole matrix this must equal nnz)
 */
int64_t oracle_decompress_rows(int elem_bytes, int64_t cols,
                               int64_t row_begin, int64_t row_end, int64_t k_begin,
                               const uint8_t *bitmap, const void *values, void *out)
{
    const uint8_t *v = (const uint8_t *)values;
    uint8_t *W = (uint8_t *)out;
    int64_t k = k_begin;
    for (int64_t i = row_begin; i < row_end; ++i) {
        for (int64_t j = 0; j < cols; ++j) {
            int64_t e = i * cols + j;
            if ((bitmap[e >> 3] >> (e & 7)) & 1) {
                memcpy(W + e * elem_bytes, v + k * elem_bytes, (size_t)elem_bytes);
                k += 1;
            } else {
                memset(W + e * elem_bytes, 0, (size_t)elem_bytes);
            }
        }
    }
    return k;
}

/* Algorithm 2 over the whole matrix. */
int64_t oracle_decompress(int elem_bytes, int64_t rows, int64_t cols,
                          const uint8_t *bitmap, const void *values, void *out)
{
    return oracle_decompress_rows(elem_bytes, cols, 0, rows, 0, bitmap, values, out);
}

/*
 * The running counter k of Algorithm 2 sampled at the start of every row:
 * row_offsets[i] = number of 1 bits among flat positions [0, i*cols).
 * rows+1 entries; the last is the total number of 1 bits.
 */
void oracle_row_offsets(int64_t rows, int64_t cols, const uint8_t *bitmap, int64_t *row_offsets)
{
    int64_t k = 0;
    for (int64_t i = 0; i < rows; ++i) {
        row_offsets[i] = k;
        for (int64_t j = 0; j < cols; ++j) {
            int64_t e = i * cols + j;
            k += (bitmap[e >> 3] >> (e & 7)) & 1;
        }
    }
    row_offsets[rows] = k;
}

/*
 * The same counter sampled every `tile` flat positions instead of every row:
 * offsets[t] = number of 1 bits among flat positions [0, min(t*tile, n)).
 * ntiles+1 entries, ntiles = ceil(n/tile).  (The paper's sequential loop never
 * needs this table; any parallel decompressor does, and this is its plain
 * definition.)
 */
void oracle_tile_offsets(int64_t n, int64_t tile, const uint8_t *bitmap, int64_t *offsets)
{
    int64_t k = 0, t = 0;
    for (int64_t e = 0; e < n; ++e) {
        if (e % tile == 0) offsets[t++] = k;
        k += (bitmap[e >> 3] >> (e & 7)) & 1;
    }
    offsets[t] = k;
}

/*
 * Row-subset decompression (the selective load Section 4.2 sketches for
 * activation sparsity): output row r of `out` (nsel x cols) is row sel[r] of
 * the full matrix.  Each selected row is Algorithm 2's inner loop started at
 * that row's own counter value row_offsets[sel[r]].
 */
void oracle_decompress_selected_rows(int elem_bytes, int64_t cols,
                                     const int64_t *sel, int64_t nsel,
                                     const int64_t *row_offsets,
                                     const uint8_t *bitmap, const void *values, void *out)
{
    const uint8_t *v = (const uint8_t *)values;
    uint8_t *W = (uint8_t *)out;
    for (int64_t r = 0; r < nsel; ++r) {
        int64_t i = sel[r];
        int64_t k = row_offsets[i];
        for (int64_t j = 0; j < cols; ++j) {
            int64_t e = i * cols + j;
            uint8_t *dst = W + (r * cols + j) * elem_bytes;
            if ((bitmap[e >> 3] >> (e & 7)) & 1) {
                memcpy(dst, v + k * elem_bytes, (size_t)elem_bytes);
                k += 1;
            } else {
                memset(dst, 0, (size_t)elem_bytes);
            }
        }
    }
}

/*
 * IEEE 754 binary16 -> double, exact (every binary16 value is a double).
 * sign 1 bit, exponent 5 bits (bias 15), fraction 10 bits; exponent 0 is zero or
 * subnormal (fraction * 2^-24), exponent 31 is Inf (fraction 0) or NaN.
 */
double oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int exp = (h >> 10) & 0x1F;
    int frac = h & 0x3FF;
    double mag;
    if (exp == 0) {
        mag = (double)frac / 16777216.0; /* frac * 2^-24 */
    } else if (exp == 31) {
        if (frac == 0) {
            mag = 1.0 / 0.0;
        } else {
            double nan = 0.0 / 0.0;
            return nan;
        }
    } else {
        /* (1 + frac/1024) * 2^(exp-15) */
        mag = 1.0 + (double)frac / 1024.0;
        int e = exp - 15;
        while (e > 0) { mag *= 2.0; --e; }
        while (e < 0) { mag *= 0.5; ++e; }
    }
    return sign ? -mag : mag;
}

void oracle_half_to_double_array(const uint16_t *h, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = oracle_half_to_double(h[i]);
}

/*
 * The dense matrix-vector product the decompressed weight is used for (the paper's
 * linear operations at batch 1, Section 3.1; computing on the compressed form
 * directly is the direction Section 7 "Efficient Compute Unit" points to):
 *     y[i] = sum_j W[i][j] * x[j]
 * with W the output of Algorithm 2 (fp16 elements), x fp16, everything converted
 * exactly to double and accumulated in double, j ascending.  Positions whose bit
 * is 0 hold +0.0 and take part in the sum like any other element, exactly as in a
 * product with the dense matrix (so a non-finite x[j] propagates the same way).
 */
void oracle_gemv_f16(int64_t rows, int64_t cols, const uint8_t *bitmap, const uint16_t *values,
                     const uint16_t *x, double *y)
{
    int64_t k = 0;
    for (int64_t i = 0; i < rows; ++i) {
        double acc = 0.0;
        for (int64_t j = 0; j < cols; ++j) {
            int64_t e = i * cols + j;
            double w;
            if ((bitmap[e >> 3] >> (e & 7)) & 1) {
                w = oracle_half_to_double(values[k]);
                k += 1;
            } else {
                w = 0.0;
            }
            acc += w * oracle_half_to_double(x[j]);
        }
        y[i] = acc;
    }
}

/*
 * The same product for a small batch of right-hand sides (the linear operation on a few
 * tokens at once; Section 7's "Efficient Compute Unit" asks for computing on the sparse
 * weight directly):
 *     y[b][i] = sum_j W[i][j] * x[b][j]        b = 0 .. nb-1
 * over the rows [row_begin, row_end) of W.  W is given DENSE, as the output of Algorithm 2
 * (oracle_decompress); this routine is only the textbook triple loop on it, every fp16
 * value converted exactly to double, sums in double, j ascending.
 *
 * dense   rows x cols fp16 patterns, row-major (the oracle's own decompressed matrix)
 * x       nb x cols fp16 patterns, each right-hand side contiguous
 * y       out, nb x rows doubles (y[b*rows + i]); only rows [row_begin,row_end) are written
 */
void oracle_gemm_f16_rows(int64_t rows, int64_t cols, int64_t row_begin, int64_t row_end,
                          const uint16_t *dense, const uint16_t *x, int64_t nb, double *y)
{
    for (int64_t b = 0; b < nb; ++b) {
        for (int64_t i = row_begin; i < row_end; ++i) {
            double acc = 0.0;
            for (int64_t j = 0; j < cols; ++j)
                acc += oracle_half_to_double(dense[i * cols + j]) * oracle_half_to_double(x[b * cols + j]);
            y[b * rows + i] = acc;
        }
    }
}
