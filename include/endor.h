/*
 * endor.h -- C ABI of the MI355X (gfx950) library for the Endor bitmap sparse
 * format: host-side compression and on-GPU decompression of an unstructured-
 * sparse weight matrix.
 *
 * THE FORMAT (paper: Figure "Sparse format" and Section 4.1; Algorithm 1 and
 * Algorithm 2).  A rows x cols matrix W of 16-bit elements (fp16 in the paper;
 * the library treats them as opaque bit patterns) is stored as
 *
 *   bitmap   one bit per element, a single 1-d bit vector over the row-major
 *            flat index e = i*cols + j.  Bit e is bit (e & 7) of byte (e >> 3),
 *            i.e. bit (e & 63) of little-endian 64-bit word (e >> 6).  There is
 *            no per-row padding.  The buffer is endor_bitmap_bytes() long
 *            (ceil(rows*cols/64) whole 64-bit words); pad bits past rows*cols
 *            are written as 0 by endor_compress and ignored by everything else.
 *   values   the elements whose bit is 1, in row-major order, packed; nnz of
 *            them (nnz == number of 1 bits).
 *
 * An element is "non-zero" when its bit pattern is not all zero, so -0.0,
 * subnormals, Inf and NaN are values like any other and a round trip is exact
 * bit for bit.  Decompression writes the all-zero pattern where the bit is 0 and
 * never inspects the values it places.
 *
 * CONVENTIONS.  Every function returns an endor_status (0 = ok); none throws,
 * aborts or prints.  The library never allocates device memory and never frees
 * or keeps caller memory; it has no mutable global state (one exception, stated
 * there: the fixed device array of endor_decompress_batch_static).  The host
 * entry points (endor_compress*, endor_build_offsets_host) use temporary host
 * memory and worker threads and report ENDOR_ERR_HOST if they cannot get them;
 * endor_pipeline_init creates HIP events, endor_pipeline_destroy releases them.
 * "host" pointers are ordinary CPU memory; "device" pointers are memory the
 * current HIP device can address: device memory, or pinned host memory from
 * hipHostMalloc (the kernels then fetch the blob across the host link
 * themselves: measured 54 GB/s against 57 GB/s for the copy engine).  Device entry
 * points only enqueue work on `stream` (a hipStream_t passed as void*, NULL = the
 * default stream) and return without synchronising; argument errors are found
 * on the host before anything is launched.  rows == 0 or cols == 0 is valid and
 * does nothing.  rows*cols must be below 2^34.
 *
 * Alignment: d_bitmap 8 bytes.  d_values 2 bytes.  d_dense 2 bytes; 16-byte
 * alignment (any torch allocation) selects the fast store path.  Workspace
 * 256 bytes.
 *
 * WORKSPACE.  Parallel decompression needs, for every tile of ENDOR_TILE_ELEMS
 * consecutive flat positions, the number of 1 bits before it (the value the
 * running counter k of Algorithm 2 has when it reaches the tile).  That table is
 * built on the device into a caller-provided workspace of
 * endor_workspace_bytes() bytes.  Calls that overlap in time need distinct
 * workspaces.  The table depends only on the bitmap, so a caller that
 * decompresses the same matrix repeatedly (every generated token, in offloaded
 * inference) may build it once with endor_build_offsets and then call the
 * *_with_offsets entry points.
 */
#ifndef ENDOR_H_
#define ENDOR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int endor_status;
enum {
    ENDOR_OK = 0,
    ENDOR_ERR_INVALID_ARG = 1,      /* NULL pointer, negative size, misaligned buffer, count out of range */
    ENDOR_ERR_BUFFER_TOO_SMALL = 2, /* values_capacity, workspace_bytes or the static scratch array too small */
    ENDOR_ERR_UNSUPPORTED = 3,      /* rows*cols >= 2^34 */
    ENDOR_ERR_HIP = 4,              /* a HIP launch or API call failed */
    ENDOR_ERR_HOST = 5,             /* host memory or a host thread could not be obtained */
    ENDOR_ERR_NNZ_MISMATCH = 6      /* written by endor_check_batch: nnz differs from the number of 1 bits */
};

/* Elements per tile of the device offset table (fixed; part of the workspace layout). */
#define ENDOR_TILE_ELEMS 4096
/* Most matrices one batched launch takes; endor_decompress_batch splits longer lists itself. */
#define ENDOR_MAX_BATCH 16

/* One compressed matrix and where to put its dense form.  All pointers are device pointers. */
typedef struct endor_matrix {
    int64_t rows;
    int64_t cols;
    const uint8_t *d_bitmap;  /* endor_bitmap_bytes(rows, cols) bytes */
    const uint16_t *d_values; /* nnz elements */
    int64_t nnz;              /* number of packed values; reads never go past it */
    uint16_t *d_dense;        /* out: rows*cols elements, row-major, contiguous */
} endor_matrix;

/* Human-readable name of a status code.  Static storage. */
const char *endor_status_string(endor_status s);

/* Bytes of the bitmap buffer of a rows x cols matrix: 8 * ceil(rows*cols/64)
 * (Section 4.1's rows*cols/8, rounded up to whole 64-bit words).  0 on bad sizes. */
size_t endor_bitmap_bytes(int64_t rows, int64_t cols);

/* Bytes of device workspace one matrix needs (a multiple of 256).  0 on bad sizes. */
size_t endor_workspace_bytes(int64_t rows, int64_t cols);

/* Bytes of device workspace a batch needs: the sum over its matrices.  Only rows
 * and cols of each entry are read.  0 on bad arguments. */
size_t endor_batch_workspace_bytes(const endor_matrix *mats, int count);

/*
 * HOST.  Algorithm 1 (Section 4.1, "Compression"): walk W in row-major order,
 * append every non-zero element to `values` and its bit to `bitmap`.
 *
 *   dense            in, host: rows*cols elements, row-major, contiguous
 *   bitmap           out, host: endor_bitmap_bytes(rows, cols) bytes, fully written
 *   values           out, host: room for values_capacity elements; may be NULL with
 *                    values_capacity 0 for a counting pass (bitmap, row_offsets and
 *                    *nnz_out are still produced)
 *   row_offsets      out, host, or NULL: rows+1 entries, row_offsets[i] = number of
 *                    non-zeros in rows before i, row_offsets[rows] = nnz
 *   nnz_out          out, host, or NULL: number of non-zeros
 *
 * ENDOR_ERR_BUFFER_TOO_SMALL if values != NULL and nnz > values_capacity; then
 * bitmap, row_offsets and *nnz_out are valid and values is untouched.
 * Runs on several host threads; returns when done.
 */
endor_status endor_compress(const uint16_t *dense, int64_t rows, int64_t cols,
                            uint8_t *bitmap, uint16_t *values, int64_t values_capacity,
                            int64_t *row_offsets, int64_t *nnz_out);

/*
 * DEVICE.  Build the tile offset table of one bitmap into d_workspace (the
 * counter k of Algorithm 2 sampled every ENDOR_TILE_ELEMS positions), and, if
 * d_row_offsets is not NULL, also the rows+1 per-row offsets
 * (d_row_offsets[i] = number of 1 bits before flat position i*cols;
 * d_row_offsets[rows] = total number of 1 bits, which a caller can compare with
 * nnz to validate a blob).
 */
endor_status endor_build_offsets(int64_t rows, int64_t cols, const uint8_t *d_bitmap,
                                 void *d_workspace, size_t workspace_bytes,
                                 int64_t *d_row_offsets, void *stream);

/*
 * HOST.  The same table built on the host, e.g. once at compression time (the paper
 * compresses before inference, Section 4.1 "Compression"), into a host buffer of
 * endor_workspace_bytes() bytes that is then copied to the device next to the blob and
 * used with the *_with_offsets entry points; no device pass over the bitmap is needed
 * then.  Every table entry equals what endor_build_offsets writes.
 */
endor_status endor_build_offsets_host(int64_t rows, int64_t cols, const uint8_t *bitmap,
                                      void *workspace, size_t workspace_bytes);

/*
 * DEVICE.  Algorithm 2 (Section 4.1, "Decompression") in parallel form: every one
 * of the rows*cols output elements is written exactly once, with the next unread
 * value where the bit is 1 and the all-zero pattern where it is 0.  Builds the
 * offset table into d_workspace first (same work as endor_build_offsets without
 * row offsets), then expands.
 */
endor_status endor_decompress(int64_t rows, int64_t cols,
                              const uint8_t *d_bitmap, const uint16_t *d_values, int64_t nnz,
                              void *d_workspace, size_t workspace_bytes,
                              uint16_t *d_dense, void *stream);

/* DEVICE.  As endor_decompress, but d_workspace already holds the table that
 * endor_build_offsets (or an earlier endor_decompress) wrote for this bitmap. */
endor_status endor_decompress_with_offsets(int64_t rows, int64_t cols,
                                           const uint8_t *d_bitmap, const uint16_t *d_values,
                                           int64_t nnz,
                                           const void *d_workspace, size_t workspace_bytes,
                                           uint16_t *d_dense, void *stream);

/*
 * DEVICE.  Decompress `count` matrices (e.g. all linear weights of one decoder
 * layer) with one pair of launches per ENDOR_MAX_BATCH matrices instead of one
 * pair per matrix.  `mats` is a HOST array, read before the call returns.
 * Matrix m uses the workspace slice that starts at the sum of
 * endor_workspace_bytes() of the matrices before it.
 */
endor_status endor_decompress_batch(const endor_matrix *mats, int count,
                                    void *d_workspace, size_t workspace_bytes, void *stream);

/* DEVICE.  Batch form of endor_build_offsets (no row offsets) and of
 * endor_decompress_with_offsets, same workspace slicing as endor_decompress_batch. */
endor_status endor_build_offsets_batch(const endor_matrix *mats, int count,
                                       void *d_workspace, size_t workspace_bytes, void *stream);
endor_status endor_decompress_batch_with_offsets(const endor_matrix *mats, int count,
                                                 const void *d_workspace, size_t workspace_bytes,
                                                 void *stream);

/*
 * DEVICE.  endor_decompress_batch for callers that cannot allocate device memory and have
 * no workspace to pass: code running under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  The offset tables go into a fixed array of
 * ENDOR_STATIC_SCRATCH_BYTES bytes of device memory that is part of the library's code
 * object (each GPU the library runs on holds its own copy until the process ends), so the
 * call takes no workspace and performs no allocation of any kind; apart from resolving the
 * array's address on its first call on a device it only enqueues the same two kernels as
 * endor_decompress_batch.  Limit: the batch's endor_batch_workspace_bytes() must not exceed
 * ENDOR_STATIC_SCRATCH_BYTES (about 4 * 2^30 elements in total), else
 * ENDOR_ERR_BUFFER_TOO_SMALL and nothing is launched.  Every call on a GPU shares that GPU's
 * array: calls that overlap in time on one GPU (different streams, or different host threads)
 * race on it; calls on one stream are ordered and safe.  The array keeps the last call's
 * tables; nothing in it needs clearing between calls.
 */
#define ENDOR_STATIC_SCRATCH_BYTES (4u << 20)
endor_status endor_decompress_batch_static(const endor_matrix *mats, int count, void *stream);

/*
 * 8-BIT ELEMENTS (Section 4.2, joint application with quantization): the same bitmap,
 * one byte per value; the compressed size becomes rows*cols/8 + nnz bytes.  The offset
 * table depends on the bitmap only, so endor_build_offsets, endor_workspace_bytes and
 * endor_batch_workspace_bytes (which read rows and cols only) serve both widths.
 * Arguments, alignment (1 byte for values and dense; 16 for the fast store path) and
 * errors are as for the 16-bit entry points of the same name.
 */
typedef struct endor_matrix_u8 {
    int64_t rows;
    int64_t cols;
    const uint8_t *d_bitmap;
    const uint8_t *d_values; /* nnz bytes */
    int64_t nnz;
    uint8_t *d_dense;        /* out: rows*cols bytes */
} endor_matrix_u8;

endor_status endor_compress_u8(const uint8_t *dense, int64_t rows, int64_t cols,
                               uint8_t *bitmap, uint8_t *values, int64_t values_capacity,
                               int64_t *row_offsets, int64_t *nnz_out);
endor_status endor_decompress_u8(int64_t rows, int64_t cols,
                                 const uint8_t *d_bitmap, const uint8_t *d_values, int64_t nnz,
                                 void *d_workspace, size_t workspace_bytes,
                                 uint8_t *d_dense, void *stream);
endor_status endor_decompress_u8_with_offsets(int64_t rows, int64_t cols,
                                              const uint8_t *d_bitmap, const uint8_t *d_values,
                                              int64_t nnz,
                                              const void *d_workspace, size_t workspace_bytes,
                                              uint8_t *d_dense, void *stream);
endor_status endor_decompress_batch_u8(const endor_matrix_u8 *mats, int count,
                                       void *d_workspace, size_t workspace_bytes, void *stream);
endor_status endor_decompress_batch_u8_with_offsets(const endor_matrix_u8 *mats, int count,
                                                    const void *d_workspace, size_t workspace_bytes,
                                                    void *stream);

/*
 * DEVICE.  Row-subset decompression: the selective load that Section 4.2 sketches for
 * activation sparsity (only the rows of an up-projection whose neurons are predicted
 * active are needed).  Output row r (of nsel) is row d_sel[r] of the matrix; the values
 * of a row start at d_row_offsets[row], the per-row table that endor_compress emits on
 * the host (copy it to the device) or endor_build_offsets builds on the device.
 * d_sel and d_row_offsets are device arrays of int64.  Rows may repeat and come in any
 * order.  An index outside [0, rows) leaves its output row untouched.  No workspace.
 * d_out: nsel*cols elements; 16-byte alignment with a row pitch that is a multiple of
 * 16 bytes selects the fast store path.  nsel*cols must be below 2^34.
 */
endor_status endor_decompress_rows(int64_t rows, int64_t cols,
                                   const uint8_t *d_bitmap, const uint16_t *d_values, int64_t nnz,
                                   const int64_t *d_row_offsets,
                                   const int64_t *d_sel, int64_t nsel,
                                   uint16_t *d_out, void *stream);
endor_status endor_decompress_rows_u8(int64_t rows, int64_t cols,
                                      const uint8_t *d_bitmap, const uint8_t *d_values, int64_t nnz,
                                      const int64_t *d_row_offsets,
                                      const int64_t *d_sel, int64_t nsel,
                                      uint8_t *d_out, void *stream);

/*
 * DEVICE.  Algorithm 1 on the GPU (the paper runs it on the host, before inference;
 * Section 4.1 "Compression"): d_dense (rows*cols elements, device) is turned into
 * d_bitmap (endor_bitmap_bytes, fully written, pad bits zero) and d_values (packed
 * non-zeros in row-major order).  The number of non-zeros is only known on the device:
 * it is written to *d_nnz_out (device int64, required), and no value is ever written at
 * or past values_capacity, so a caller that cannot bound nnz runs with capacity 0 first
 * (bitmap, offsets and *d_nnz_out are still produced) or passes capacity rows*cols.
 * d_row_offsets (device, rows+1 entries) is optional.  Afterwards d_workspace holds the
 * tile offset table of the new bitmap, ready for the *_with_offsets entry points.
 * Alignment as elsewhere; a 16-byte aligned d_dense selects the fast load path.
 */
endor_status endor_compress_device(int64_t rows, int64_t cols, const uint16_t *d_dense,
                                   uint8_t *d_bitmap, uint16_t *d_values, int64_t values_capacity,
                                   void *d_workspace, size_t workspace_bytes,
                                   int64_t *d_row_offsets, int64_t *d_nnz_out, void *stream);
endor_status endor_compress_device_u8(int64_t rows, int64_t cols, const uint8_t *d_dense,
                                      uint8_t *d_bitmap, uint8_t *d_values, int64_t values_capacity,
                                      void *d_workspace, size_t workspace_bytes,
                                      int64_t *d_row_offsets, int64_t *d_nnz_out, void *stream);

/*
 * DEVICE.  Column-subset decompression, the other half of Section 4.2's selective load (the
 * columns of a down projection that belong to active neurons): d_out is rows x nsel,
 * d_out[i][q] = W[i][d_sel[q]].  One rank query per row and selected column, answered from
 * the bitmap and d_row_offsets.  Columns may repeat and come in any order; an index outside
 * [0, cols) leaves its output column untouched.  cols <= 2^18; rows*nsel < 2^34.
 * d_sel, d_row_offsets: device int64 arrays.  No workspace.
 */
endor_status endor_decompress_cols(int64_t rows, int64_t cols,
                                   const uint8_t *d_bitmap, const uint16_t *d_values, int64_t nnz,
                                   const int64_t *d_row_offsets,
                                   const int64_t *d_sel, int64_t nsel,
                                   uint16_t *d_out, void *stream);
endor_status endor_decompress_cols_u8(int64_t rows, int64_t cols,
                                      const uint8_t *d_bitmap, const uint8_t *d_values, int64_t nnz,
                                      const int64_t *d_row_offsets,
                                      const int64_t *d_sel, int64_t nsel,
                                      uint8_t *d_out, void *stream);

/*
 * DEVICE.  Fused consumer: y = W x computed straight from the compressed form, without
 * writing the dense matrix (the batch-1 linear operation the paper's workload runs on the
 * decompressed weight, Section 3.1; computing on the sparse form is the direction of
 * Section 7, "Efficient Compute Unit").  W: fp16 values; x: cols fp16 values (device);
 * y: rows fp32 results (device), y[i] = sum_j W[i][j]*x[j] with fp16 products exact and
 * accumulation in fp32.  Elements whose bit is 0 enter as +0.0, as from the dense matrix.
 * d_row_offsets as for endor_decompress_rows.  16-byte aligned d_x selects the fast path.
 */
endor_status endor_gemv_f16(int64_t rows, int64_t cols,
                            const uint8_t *d_bitmap, const uint16_t *d_values, int64_t nnz,
                            const int64_t *d_row_offsets,
                            const uint16_t *d_x, float *d_y, void *stream);

/*
 * DEVICE.  Fused consumer for a small batch: Y = X W^T for nb <= ENDOR_GEMM_MAX_BATCH
 * right-hand sides, straight from the compressed form, on the matrix cores (Section 7,
 * "Efficient Compute Unit": compute on the sparse weight; Section 3.1: the linear operation
 * itself).  The expansion of W is done once and shared by all right-hand sides.
 *   d_x      nb vectors of cols fp16 values; vector b starts at d_x + b*ldx (ldx >= cols)
 *   d_y      out, nb x rows fp32: d_y[b*rows + i] = sum_j W[i][j] * x_b[j]; fp16 products are
 *            exact, sums are fp32 (32 products per matrix instruction); elements whose bit is
 *            0 enter as +0.0, fp16 subnormals count in full
 *   d_workspace   the tile offset table of this bitmap (endor_build_offsets or any
 *            endor_decompress* call wrote it): it gives every wave its starting point
 *   d_scratch     endor_gemm_scratch_bytes(rows, cols, nb) bytes (256-byte aligned; may be NULL
 *            when that is 0): partial sums of the column ranges the work is split into; they
 *            are added in a fixed order, so results are reproducible from run to run
 * A 16-byte aligned d_x with ldx a multiple of 8 selects the fast load path.  rows < 2^31.
 */
#define ENDOR_GEMM_MAX_BATCH 16
size_t endor_gemm_scratch_bytes(int64_t rows, int64_t cols, int nb);
endor_status endor_gemm_f16(int64_t rows, int64_t cols,
                            const uint8_t *d_bitmap, const uint16_t *d_values, int64_t nnz,
                            const void *d_workspace, size_t workspace_bytes,
                            const uint16_t *d_x, int64_t ldx, int nb, float *d_y,
                            void *d_scratch, size_t scratch_bytes, void *stream);

/*
 * DEVICE.  Check mode (the end condition of Algorithm 2: its counter k must equal the
 * number of packed values).  For each matrix of the batch, compare its nnz with the
 * number of 1 bits of its bitmap as recorded in the offset tables that
 * endor_decompress_batch / endor_build_offsets_batch wrote into d_workspace, and write
 * ENDOR_OK or ENDOR_ERR_NNZ_MISMATCH to d_status[i] (device, `count` 32-bit words).  One
 * small launch on `stream`, no synchronisation; the caller reads d_status whenever it next
 * synchronises anyway.  Decompression of a blob with a wrong nnz is still memory-safe
 * (values past nnz read as zero); this call is how a caller finds out.
 */
endor_status endor_check_batch(const endor_matrix *mats, int count,
                               const void *d_workspace, size_t workspace_bytes,
                               int32_t *d_status, void *stream);

/*
 * HOST -> DEVICE transfer overlapped with decompression (the paper's inference-time
 * order for a CPU-mapped layer, Section 4.1 "Decompression": the compressed weight
 * is copied from host memory to GPU memory and decompressed there; Section 6 notes
 * that the smaller transfers make overlap with other GPU work worthwhile).
 *
 * One blob = one compressed matrix (or a block of whole rows of one, see
 * endor_row_block) in HOST memory, preferably pinned (hipHostMalloc / torch
 * pin_memory), and the device address its dense form goes to.  elem_bytes is 2 for
 * fp16 values and 1 for the 8-bit variant of Section 4.2 (whose transfer saving is
 * what Section 5.4 measures).  If h_values lies exactly
 * align256(endor_bitmap_bytes(rows, cols)) bytes after h_bitmap (align256 = round up to a
 * multiple of 256), the blob crosses the link in one copy instead of two.
 */
typedef struct endor_host_blob {
    int64_t rows;
    int64_t cols;
    const uint8_t *h_bitmap; /* host: endor_bitmap_bytes(rows, cols) bytes readable */
    const void *h_values;    /* host: nnz elements of elem_bytes bytes */
    int64_t nnz;
    void *d_dense;           /* device out: rows*cols elements */
    int32_t elem_bytes;      /* 2 or 1 */
    int32_t reserved;        /* 0 */
} endor_host_blob;

/* Bytes of ONE device staging slot able to hold this blob's bitmap and values
 * (each rounded up to 256 bytes).  0 on bad arguments. */
size_t endor_stage_bytes(int64_t rows, int64_t cols, int64_t nnz, int elem_bytes);

/*
 * HOST.  Row blocks: a matrix may be fed to the pipeline as several blobs of whole rows
 * [r0, r1) for finer overlap.  endor_row_block_cuts chooses the block boundaries:
 * `nblocks`+1 non-decreasing row indices from 0 to rows, each a multiple of the smallest
 * row count whose bits fill whole 64-bit bitmap words (so every block's bitmap starts on a
 * word boundary); blocks that come out empty are legal.  endor_row_block fills `out` for
 * rows [r0, r1) of a compressed matrix in host memory: its bitmap starts at byte
 * r0*cols/8 of the matrix's, its values at element row_offsets[r0], nnz =
 * row_offsets[r1] - row_offsets[r0], d_dense = d_dense + r0*cols elements.  The bits
 * after the block's last row in its final bitmap word belong to the next rows and are
 * ignored by decompression, as pad bits are.  ENDOR_ERR_INVALID_ARG if r0*cols is not a
 * multiple of 64 or the range is not inside the matrix.
 */
endor_status endor_row_block_cuts(int64_t rows, int64_t cols, int nblocks, int64_t *cuts);
endor_status endor_row_block(int64_t rows, int64_t cols, int elem_bytes,
                             const uint8_t *h_bitmap, const void *h_values,
                             const int64_t *row_offsets, int64_t r0, int64_t r1,
                             void *d_dense, endor_host_blob *out);

/*
 * The pipeline's state: three device staging slots and workspaces (caller-owned memory),
 * two streams, and the events that order a slot's copy before its decompression and its
 * decompression before the next copy into it.  The state lives across calls, so a call may
 * follow an earlier one whose work is still running: the same events keep the slots safe.
 * One endor_pipeline must not be used by two host threads at once.
 */
#define ENDOR_PIPELINE_SLOTS 3
typedef struct endor_pipeline {
    void *d_stage[ENDOR_PIPELINE_SLOTS];
    void *d_workspace[ENDOR_PIPELINE_SLOTS];
    size_t stage_bytes;
    size_t workspace_bytes;
    void *copy_stream;    /* hipStream_t */
    void *copy_stream2;   /* hipStream_t or NULL: if set, blobs alternate between the two copy streams */
    void *compute_stream; /* hipStream_t */
    void *copied[ENDOR_PIPELINE_SLOTS]; /* hipEvent_t: the slot's blob has arrived */
    void *freed[ENDOR_PIPELINE_SLOTS];  /* hipEvent_t: the slot's decompression has finished reading it */
    uint32_t next_slot;
    uint32_t slots_used;  /* bit b: freed[b] has been recorded at least once */
    uint64_t blobs_done;  /* blobs enqueued so far */
} endor_pipeline;

/* Fill *p and create its six events (disable-timing).  copy_stream and compute_stream must
 * be non-NULL; all streams distinct and of default priority.  copy_stream2 may be NULL.  With
 * two copy streams consecutive blobs travel on alternating streams, so the next copy is
 * already queued on a second copy engine when one ends (on MI355X consecutive copies on ONE
 * stream leave the link idle for 20-50 us each time; whole matrices, few and large, do better
 * on one stream, many row blocks on two).  Each d_stage[b] must hold stage_bytes bytes (the
 * largest endor_stage_bytes of the blobs to come), each d_workspace[b] workspace_bytes
 * (the largest endor_workspace_bytes); all 256-byte aligned and distinct. */
endor_status endor_pipeline_init(endor_pipeline *p,
                                 void *const d_stage[ENDOR_PIPELINE_SLOTS], size_t stage_bytes,
                                 void *const d_workspace[ENDOR_PIPELINE_SLOTS], size_t workspace_bytes,
                                 void *copy_stream, void *copy_stream2, void *compute_stream);

/* Destroy the events.  Work already enqueued still completes. */
endor_status endor_pipeline_destroy(endor_pipeline *p);

/*
 * Enqueue `count` blobs: on copy_stream blob k is copied into the next staging slot
 * (hipMemcpyAsync) while compute_stream decompresses earlier blobs out of the other slots.
 * Creates nothing, allocates nothing, and returns after enqueueing; the dense outputs are
 * complete when compute_stream has drained.  Blobs larger than the slots are refused with
 * ENDOR_ERR_BUFFER_TOO_SMALL before anything is enqueued.
 */
endor_status endor_h2d_decompress_pipeline(endor_pipeline *p, const endor_host_blob *blobs, int count);

#ifdef __cplusplus
}
#endif
#endif /* ENDOR_H_ */
