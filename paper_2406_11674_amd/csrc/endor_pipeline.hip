// Host-to-device copy of compressed blobs overlapped with their decompression:
// two HIP streams, three device staging slots, events between them.  This is the
// transfer step the paper places before GPU decompression (Section 4.1,
// "Decompression"), arranged so that the PCIe copy of blob k+1 runs under the
// decompression of blob k.
//
// What the copy engine dislikes (measured with a copy/kernel trace on MI355X): every
// separate hipMemcpyAsync costs about 30 us of idle link, and every wait of the copy
// stream on an event of the compute stream about 70 us.  So a blob whose bitmap and
// values are adjacent in host memory goes over in ONE copy, and the copy stream only
// waits for a slot's previous decompression when hipEventQuery says it has not finished
// yet (with three slots it practically always has: decompression is some thirty times
// faster than the link).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>

#include "endor.h"
#include "endor_layout.h"

namespace {

using endor_layout::align256;

struct BlobView {
    int64_t n = 0;
    size_t bitmap_bytes = 0;
    size_t value_bytes = 0;
    bool adjacent = false;  // values start align256(bitmap_bytes) after the bitmap in host memory
};

endor_status view_of(const endor_host_blob &B, BlobView *v) {
    if (B.rows < 0 || B.cols < 0 || B.nnz < 0) return ENDOR_ERR_INVALID_ARG;
    if (B.elem_bytes != 1 && B.elem_bytes != 2) return ENDOR_ERR_INVALID_ARG;
    v->n = (B.rows == 0 || B.cols == 0) ? 0 : B.rows * B.cols;
    if (v->n == 0) return ENDOR_OK;
    v->bitmap_bytes = endor_bitmap_bytes(B.rows, B.cols);
    if (v->bitmap_bytes == 0) return ENDOR_ERR_UNSUPPORTED;
    if (B.nnz > v->n || !B.h_bitmap || !B.d_dense || (B.nnz > 0 && !B.h_values)) return ENDOR_ERR_INVALID_ARG;
    v->value_bytes = static_cast<size_t>(B.elem_bytes) * static_cast<size_t>(B.nnz);
    v->adjacent = B.nnz > 0 && static_cast<const char *>(B.h_values) ==
                                   reinterpret_cast<const char *>(B.h_bitmap) + align256(v->bitmap_bytes);
    return ENDOR_OK;
}

}  // namespace

extern "C" size_t endor_stage_bytes(int64_t rows, int64_t cols, int64_t nnz, int elem_bytes) {
    if (nnz < 0 || (elem_bytes != 1 && elem_bytes != 2)) return 0;
    if (rows == 0 || cols == 0) return nnz == 0 ? 256 : 0;
    const size_t bm = endor_bitmap_bytes(rows, cols);
    if (bm == 0 || nnz > rows * cols) return 0;
    return align256(bm) + align256(static_cast<size_t>(elem_bytes) * static_cast<size_t>(nnz));
}

extern "C" endor_status endor_pipeline_init(endor_pipeline *p, void *const d_stage[ENDOR_PIPELINE_SLOTS],
                                            size_t stage_bytes, void *const d_workspace[ENDOR_PIPELINE_SLOTS],
                                            size_t workspace_bytes, void *copy_stream, void *copy_stream2,
                                            void *compute_stream) {
    if (!p || !d_stage || !d_workspace) return ENDOR_ERR_INVALID_ARG;
    if (!copy_stream || !compute_stream || copy_stream == compute_stream) return ENDOR_ERR_INVALID_ARG;
    if (copy_stream2 && (copy_stream2 == copy_stream || copy_stream2 == compute_stream)) return ENDOR_ERR_INVALID_ARG;
    for (int b = 0; b < ENDOR_PIPELINE_SLOTS; ++b) {
        if (!d_stage[b] || (reinterpret_cast<uintptr_t>(d_stage[b]) & 255)) return ENDOR_ERR_INVALID_ARG;
        if (!d_workspace[b] || (reinterpret_cast<uintptr_t>(d_workspace[b]) & 255)) return ENDOR_ERR_INVALID_ARG;
        for (int a = 0; a < b; ++a)
            if (d_stage[a] == d_stage[b] || d_workspace[a] == d_workspace[b]) return ENDOR_ERR_INVALID_ARG;
    }
    std::memset(p, 0, sizeof(*p));
    for (int b = 0; b < ENDOR_PIPELINE_SLOTS; ++b) {
        p->d_stage[b] = d_stage[b];
        p->d_workspace[b] = d_workspace[b];
    }
    p->stage_bytes = stage_bytes;
    p->workspace_bytes = workspace_bytes;
    p->copy_stream = copy_stream;
    p->copy_stream2 = copy_stream2;
    p->compute_stream = compute_stream;
    for (int b = 0; b < ENDOR_PIPELINE_SLOTS; ++b) {
        hipEvent_t c = nullptr, f = nullptr;
        if (hipEventCreateWithFlags(&c, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&f, hipEventDisableTiming) != hipSuccess) {
            if (c) (void)hipEventDestroy(c);
            endor_pipeline_destroy(p);
            return ENDOR_ERR_HIP;
        }
        p->copied[b] = c;
        p->freed[b] = f;
    }
    return ENDOR_OK;
}

extern "C" endor_status endor_pipeline_destroy(endor_pipeline *p) {
    if (!p) return ENDOR_ERR_INVALID_ARG;
    endor_status st = ENDOR_OK;
    for (int b = 0; b < ENDOR_PIPELINE_SLOTS; ++b) {
        // destroying a recorded event is legal; its resources go once the work has passed it
        if (p->copied[b] && hipEventDestroy(static_cast<hipEvent_t>(p->copied[b])) != hipSuccess) st = ENDOR_ERR_HIP;
        if (p->freed[b] && hipEventDestroy(static_cast<hipEvent_t>(p->freed[b])) != hipSuccess) st = ENDOR_ERR_HIP;
        p->copied[b] = p->freed[b] = nullptr;
    }
    p->slots_used = 0;
    return st;
}

extern "C" endor_status endor_h2d_decompress_pipeline(endor_pipeline *p, const endor_host_blob *blobs, int count) {
    if (!p || count < 0 || (count > 0 && !blobs)) return ENDOR_ERR_INVALID_ARG;
    if (count == 0) return ENDOR_OK;
    for (int b = 0; b < ENDOR_PIPELINE_SLOTS; ++b)
        if (!p->copied[b] || !p->freed[b]) return ENDOR_ERR_INVALID_ARG;  // not initialised, or destroyed

    // validate every blob before anything is enqueued
    for (int k = 0; k < count; ++k) {
        BlobView v;
        const endor_status st = view_of(blobs[k], &v);
        if (st != ENDOR_OK) return st;
        if (v.n == 0) continue;
        if (endor_stage_bytes(blobs[k].rows, blobs[k].cols, blobs[k].nnz, blobs[k].elem_bytes) > p->stage_bytes)
            return ENDOR_ERR_BUFFER_TOO_SMALL;
        if (endor_workspace_bytes(blobs[k].rows, blobs[k].cols) > p->workspace_bytes) return ENDOR_ERR_BUFFER_TOO_SMALL;
    }

    hipStream_t ks = static_cast<hipStream_t>(p->compute_stream);
    for (int k = 0; k < count; ++k) {
        const endor_host_blob &B = blobs[k];
        BlobView v;
        view_of(B, &v);
        if (v.n == 0) continue;
        const unsigned b = p->next_slot;
        p->next_slot = (b + 1) % ENDOR_PIPELINE_SLOTS;
        hipStream_t cs = static_cast<hipStream_t>((p->copy_stream2 && (p->blobs_done & 1)) ? p->copy_stream2
                                                                                             : p->copy_stream);
        ++p->blobs_done;
        hipEvent_t copied = static_cast<hipEvent_t>(p->copied[b]);
        hipEvent_t freed = static_cast<hipEvent_t>(p->freed[b]);
        char *stage = static_cast<char *>(p->d_stage[b]);
        uint8_t *d_bitmap = reinterpret_cast<uint8_t *>(stage);
        char *d_values = stage + align256(v.bitmap_bytes);

        // The copy into slot b must stay behind the decompression that last read the slot
        // (possibly enqueued by an earlier call).  Usually that one finished long ago.
        if (p->slots_used & (1u << b)) {
            const hipError_t q = hipEventQuery(freed);
            if (q == hipErrorNotReady) {
                if (hipStreamWaitEvent(cs, freed, 0) != hipSuccess) return ENDOR_ERR_HIP;
            } else if (q != hipSuccess) {
                return ENDOR_ERR_HIP;
            }
        }
        if (v.adjacent) {
            if (hipMemcpyAsync(d_bitmap, B.h_bitmap, align256(v.bitmap_bytes) + v.value_bytes, hipMemcpyHostToDevice,
                               cs) != hipSuccess)
                return ENDOR_ERR_HIP;
        } else {
            if (hipMemcpyAsync(d_bitmap, B.h_bitmap, v.bitmap_bytes, hipMemcpyHostToDevice, cs) != hipSuccess)
                return ENDOR_ERR_HIP;
            if (B.nnz > 0 &&
                hipMemcpyAsync(d_values, B.h_values, v.value_bytes, hipMemcpyHostToDevice, cs) != hipSuccess)
                return ENDOR_ERR_HIP;
        }
        if (hipEventRecord(copied, cs) != hipSuccess) return ENDOR_ERR_HIP;

        if (hipStreamWaitEvent(ks, copied, 0) != hipSuccess) return ENDOR_ERR_HIP;
        endor_status st;
        if (B.elem_bytes == 2)
            st = endor_decompress(B.rows, B.cols, d_bitmap, reinterpret_cast<const uint16_t *>(d_values), B.nnz,
                                  p->d_workspace[b], p->workspace_bytes, static_cast<uint16_t *>(B.d_dense), ks);
        else
            st = endor_decompress_u8(B.rows, B.cols, d_bitmap, reinterpret_cast<const uint8_t *>(d_values), B.nnz,
                                     p->d_workspace[b], p->workspace_bytes, static_cast<uint8_t *>(B.d_dense), ks);
        if (st != ENDOR_OK) return st;
        if (hipEventRecord(freed, ks) != hipSuccess) return ENDOR_ERR_HIP;
        p->slots_used |= 1u << b;
    }
    return ENDOR_OK;
}
