// Host-to-device copy of compressed blobs overlapped with their decompression:
// two HIP streams, two device staging buffers, events between them.  This is the
// transfer step the paper places before GPU decompression (Section 4.1,
// "Decompression"), arranged so that the PCIe copy of blob k+1 runs under the
// decompression of blob k.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "endor.h"

namespace {

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

struct EventPair {
    hipEvent_t copied = nullptr;  // blob is in the staging buffer
    hipEvent_t freed = nullptr;   // decompression has finished reading the staging buffer
    bool freed_recorded = false;
    ~EventPair() {
        // destroying a recorded event is legal; its resources go once the work has passed it
        if (copied) (void)hipEventDestroy(copied);
        if (freed) (void)hipEventDestroy(freed);
    }
};

}  // namespace

extern "C" size_t endor_stage_bytes(int64_t rows, int64_t cols, int64_t nnz) {
    if (nnz < 0) return 0;
    if (rows == 0 || cols == 0) return nnz == 0 ? 256 : 0;
    const size_t bm = endor_bitmap_bytes(rows, cols);
    if (bm == 0 || nnz > rows * cols) return 0;
    return align256(bm) + align256(2 * static_cast<size_t>(nnz));
}

extern "C" endor_status endor_h2d_decompress_pipeline(const endor_host_blob *blobs, int count,
                                                      void *const d_stage[2], size_t stage_bytes,
                                                      void *const d_workspace[2], size_t workspace_bytes,
                                                      void *copy_stream, void *compute_stream) {
    if (count < 0 || (count > 0 && !blobs)) return ENDOR_ERR_INVALID_ARG;
    if (count == 0) return ENDOR_OK;
    if (!copy_stream || !compute_stream || copy_stream == compute_stream) return ENDOR_ERR_INVALID_ARG;
    if (!d_stage || !d_workspace) return ENDOR_ERR_INVALID_ARG;
    for (int b = 0; b < 2; ++b) {
        if (!d_stage[b] || (reinterpret_cast<uintptr_t>(d_stage[b]) & 255)) return ENDOR_ERR_INVALID_ARG;
        if (!d_workspace[b] || (reinterpret_cast<uintptr_t>(d_workspace[b]) & 255)) return ENDOR_ERR_INVALID_ARG;
    }
    if (d_stage[0] == d_stage[1] || d_workspace[0] == d_workspace[1]) return ENDOR_ERR_INVALID_ARG;

    // validate every blob before anything is enqueued
    for (int k = 0; k < count; ++k) {
        const endor_host_blob &B = blobs[k];
        if (B.rows < 0 || B.cols < 0 || B.nnz < 0) return ENDOR_ERR_INVALID_ARG;
        const int64_t n = (B.rows == 0 || B.cols == 0) ? 0 : B.rows * B.cols;
        if (n == 0) continue;
        const size_t bm = endor_bitmap_bytes(B.rows, B.cols);
        if (bm == 0) return ENDOR_ERR_UNSUPPORTED;
        if (B.nnz > n || !B.h_bitmap || !B.d_dense || (B.nnz > 0 && !B.h_values)) return ENDOR_ERR_INVALID_ARG;
        if (endor_stage_bytes(B.rows, B.cols, B.nnz) > stage_bytes) return ENDOR_ERR_BUFFER_TOO_SMALL;
        if (endor_workspace_bytes(B.rows, B.cols) > workspace_bytes) return ENDOR_ERR_BUFFER_TOO_SMALL;
    }

    hipStream_t cs = static_cast<hipStream_t>(copy_stream);
    hipStream_t ks = static_cast<hipStream_t>(compute_stream);
    EventPair ev[2];
    for (int b = 0; b < 2; ++b) {
        if (hipEventCreateWithFlags(&ev[b].copied, hipEventDisableTiming) != hipSuccess) return ENDOR_ERR_HIP;
        if (hipEventCreateWithFlags(&ev[b].freed, hipEventDisableTiming) != hipSuccess) return ENDOR_ERR_HIP;
    }

    int slot = 0;
    for (int k = 0; k < count; ++k) {
        const endor_host_blob &B = blobs[k];
        const int64_t n = (B.rows == 0 || B.cols == 0) ? 0 : B.rows * B.cols;
        if (n == 0) continue;
        const int b = slot & 1;
        ++slot;
        char *stage = static_cast<char *>(d_stage[b]);
        const size_t bm = endor_bitmap_bytes(B.rows, B.cols);
        uint8_t *d_bitmap = reinterpret_cast<uint8_t *>(stage);
        uint16_t *d_values = reinterpret_cast<uint16_t *>(stage + align256(bm));

        // the copy into buffer b waits until the decompression that last read it is done
        if (ev[b].freed_recorded && hipStreamWaitEvent(cs, ev[b].freed, 0) != hipSuccess) return ENDOR_ERR_HIP;
        if (hipMemcpyAsync(d_bitmap, B.h_bitmap, bm, hipMemcpyHostToDevice, cs) != hipSuccess) return ENDOR_ERR_HIP;
        if (B.nnz > 0 &&
            hipMemcpyAsync(d_values, B.h_values, 2 * static_cast<size_t>(B.nnz), hipMemcpyHostToDevice, cs) !=
                hipSuccess)
            return ENDOR_ERR_HIP;
        if (hipEventRecord(ev[b].copied, cs) != hipSuccess) return ENDOR_ERR_HIP;

        if (hipStreamWaitEvent(ks, ev[b].copied, 0) != hipSuccess) return ENDOR_ERR_HIP;
        const endor_status st = endor_decompress(B.rows, B.cols, d_bitmap, d_values, B.nnz, d_workspace[b],
                                                 workspace_bytes, B.d_dense, ks);
        if (st != ENDOR_OK) return st;
        if (hipEventRecord(ev[b].freed, ks) != hipSuccess) return ENDOR_ERR_HIP;
        ev[b].freed_recorded = true;
    }
    return ENDOR_OK;
}
