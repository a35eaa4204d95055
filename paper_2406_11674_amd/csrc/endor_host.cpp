// Host side of the Endor library: size helpers, status strings and the
// compressor (Algorithm 1 of the paper, Section 4.1 "Compression").
//
// The compressor is the off-line step of the method: it walks the dense matrix
// in row-major order once and emits the position bitmap and the packed non-zero
// values.  Here the walk is split over host threads by ranges of 64-bit bitmap
// words: pass 1 builds the bitmap words of a range and counts its 1 bits, a
// serial prefix over the per-range counts gives each range its start in the
// value stream, pass 2 packs the values and samples the running count at every
// row start.
#include "endor.h"
#include "endor_layout.h"

#include <algorithm>
#include <cstring>
#include <new>
#include <numeric>
#include <system_error>
#include <thread>
#include <vector>

#if defined(__SSE2__)
#include <emmintrin.h>
#endif

namespace {

using endor_layout::dims_ok;

// bit i of the result = (d[i] != 0), for 64 consecutive elements
inline uint64_t nonzero_mask64(const uint16_t *d) {
#if defined(__SSE2__)
    const __m128i zero = _mm_setzero_si128();
    uint64_t m = 0;
    for (int g = 0; g < 4; ++g) {
        __m128i a = _mm_loadu_si128(reinterpret_cast<const __m128i *>(d + 16 * g));
        __m128i b = _mm_loadu_si128(reinterpret_cast<const __m128i *>(d + 16 * g + 8));
        // 0xFFFF where the element is zero; narrow to bytes, one bit per byte
        __m128i z = _mm_packs_epi16(_mm_cmpeq_epi16(a, zero), _mm_cmpeq_epi16(b, zero));
        uint64_t zeros = static_cast<uint32_t>(_mm_movemask_epi8(z));
        m |= ((~zeros) & 0xFFFFull) << (16 * g);
    }
    return m;
#else
    uint64_t m = 0;
    for (int i = 0; i < 64; ++i) m |= uint64_t(d[i] != 0) << i;
    return m;
#endif
}

// the same for 64 consecutive one-byte elements
inline uint64_t nonzero_mask64(const uint8_t *d) {
#if defined(__SSE2__)
    const __m128i zero = _mm_setzero_si128();
    uint64_t m = 0;
    for (int g = 0; g < 4; ++g) {
        __m128i a = _mm_loadu_si128(reinterpret_cast<const __m128i *>(d + 16 * g));
        uint64_t zeros = static_cast<uint32_t>(_mm_movemask_epi8(_mm_cmpeq_epi8(a, zero)));
        m |= ((~zeros) & 0xFFFFull) << (16 * g);
    }
    return m;
#else
    uint64_t m = 0;
    for (int i = 0; i < 64; ++i) m |= uint64_t(d[i] != 0) << i;
    return m;
#endif
}

template <class T>
inline uint64_t nonzero_mask_tail(const T *d, int count) {
    uint64_t m = 0;
    for (int i = 0; i < count; ++i) m |= uint64_t(d[i] != 0) << i;
    return m;
}

struct Range {
    int64_t w0, w1;    // bitmap words [w0, w1)
    int64_t ones = 0;  // 1 bits in the range
    int64_t base = 0;  // 1 bits before the range
};

// Run f(0) .. f(nthreads-1), each on a thread of its own where one can be had; parts whose
// thread cannot be created run on the calling thread instead.
template <class F>
void run_threads(int nthreads, F &&f) {
    if (nthreads <= 1) {
        f(0);
        return;
    }
    std::vector<std::thread> pool;
    pool.reserve(nthreads - 1);
    int started = 1;
    try {
        for (; started < nthreads; ++started) pool.emplace_back([&f, t = started] { f(t); });
    } catch (const std::system_error &) {
        // no more threads: parts started .. nthreads-1 are done below
    }
    f(0);
    for (int t = started; t < nthreads; ++t) f(t);
    for (auto &th : pool) th.join();
}

// The extern "C" entry points must not let an exception out (std::bad_alloc from the
// vectors, std::system_error from thread start-up).
template <class F>
endor_status no_throw(F &&f) {
    try {
        return f();
    } catch (...) {
        return ENDOR_ERR_HOST;
    }
}

}  // namespace

extern "C" const char *endor_status_string(endor_status s) {
    switch (s) {
        case ENDOR_OK: return "ok";
        case ENDOR_ERR_INVALID_ARG: return "invalid argument";
        case ENDOR_ERR_BUFFER_TOO_SMALL: return "buffer too small";
        case ENDOR_ERR_UNSUPPORTED: return "unsupported size";
        case ENDOR_ERR_HIP: return "HIP error";
        case ENDOR_ERR_HOST: return "out of host memory or threads";
        case ENDOR_ERR_NNZ_MISMATCH: return "nnz differs from the number of 1 bits";
        default: return "unknown status";
    }
}

extern "C" size_t endor_bitmap_bytes(int64_t rows, int64_t cols) {
    if (!dims_ok(rows, cols)) return 0;
    const int64_t n = rows * cols;
    return static_cast<size_t>((n + 63) / 64) * 8;
}

namespace {

template <class T>
endor_status compress_impl(const T *dense, int64_t rows, int64_t cols, uint8_t *bitmap, T *values,
                           int64_t values_capacity, int64_t *row_offsets, int64_t *nnz_out) {
    if (rows < 0 || cols < 0 || values_capacity < 0) return ENDOR_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols)) return ENDOR_ERR_UNSUPPORTED;
    const int64_t n = rows * cols;
    if (n == 0) {
        if (row_offsets) std::fill(row_offsets, row_offsets + rows + 1, int64_t(0));
        if (nnz_out) *nnz_out = 0;
        return ENDOR_OK;
    }
    if (!dense || !bitmap) return ENDOR_ERR_INVALID_ARG;
    if (!values && values_capacity != 0) return ENDOR_ERR_INVALID_ARG;

    const int64_t nwords = (n + 63) / 64;
    const int64_t full_words = n / 64;
    unsigned hw = std::thread::hardware_concurrency();
    int nthreads = static_cast<int>(std::min<int64_t>(hw ? hw : 1, std::max<int64_t>(1, nwords / 8192)));
    nthreads = std::min(nthreads, 64);
    std::vector<Range> ranges(nthreads);
    for (int t = 0; t < nthreads; ++t) {
        ranges[t].w0 = nwords * t / nthreads;
        ranges[t].w1 = nwords * (t + 1) / nthreads;
    }

    // pass 1: bitmap words and per-range counts.  The bitmap may be only byte
    // aligned on the host, so words are stored with memcpy.
    run_threads(nthreads, [&](int t) {
        Range &r = ranges[t];
        int64_t ones = 0;
        for (int64_t w = r.w0; w < r.w1; ++w) {
            uint64_t m = (w < full_words) ? nonzero_mask64(dense + 64 * w)
                                          : nonzero_mask_tail(dense + 64 * w, static_cast<int>(n - 64 * w));
            std::memcpy(bitmap + 8 * w, &m, 8);
            ones += __builtin_popcountll(m);
        }
        r.ones = ones;
    });

    int64_t nnz = 0;
    for (auto &r : ranges) {
        r.base = nnz;
        nnz += r.ones;
    }
    if (nnz_out) *nnz_out = nnz;
    const bool pack = values != nullptr && nnz <= values_capacity;

    // pass 2: pack the values of each range at its start, and sample the running
    // count at the row starts that fall into the range.
    run_threads(nthreads, [&](int t) {
        const Range &r = ranges[t];
        int64_t k = r.base;
        // first row whose start e = i*cols lies at or after the range's first element
        int64_t next_row = row_offsets ? (64 * r.w0 + cols - 1) / cols : rows;
        for (int64_t w = r.w0; w < r.w1; ++w) {
            uint64_t m;
            std::memcpy(&m, bitmap + 8 * w, 8);
            const int64_t e0 = 64 * w;
            // row starts inside this word (the entry for position rows*cols is
            // written after the loop)
            while (next_row < rows && next_row * cols < e0 + 64) {
                const int bit = static_cast<int>(next_row * cols - e0);  // 0..63
                const uint64_t below = bit ? (m & (~uint64_t(0) >> (64 - bit))) : 0;
                row_offsets[next_row] = k + __builtin_popcountll(below);
                ++next_row;
            }
            if (pack) {
                const T *d = dense + e0;
                if (m == ~uint64_t(0)) {
                    std::memcpy(values + k, d, 64 * sizeof(T));
                    k += 64;
                } else {
                    uint64_t mm = m;
                    while (mm) {
                        values[k++] = d[__builtin_ctzll(mm)];
                        mm &= mm - 1;
                    }
                }
            } else {
                k += __builtin_popcountll(m);
            }
        }
    });
    if (row_offsets) row_offsets[rows] = nnz;
    if (values != nullptr && nnz > values_capacity) return ENDOR_ERR_BUFFER_TOO_SMALL;
    return ENDOR_OK;
}

}  // namespace

extern "C" endor_status endor_compress(const uint16_t *dense, int64_t rows, int64_t cols,
                                       uint8_t *bitmap, uint16_t *values, int64_t values_capacity,
                                       int64_t *row_offsets, int64_t *nnz_out) {
    return no_throw([&] {
        return compress_impl<uint16_t>(dense, rows, cols, bitmap, values, values_capacity, row_offsets, nnz_out);
    });
}

extern "C" endor_status endor_compress_u8(const uint8_t *dense, int64_t rows, int64_t cols,
                                          uint8_t *bitmap, uint8_t *values, int64_t values_capacity,
                                          int64_t *row_offsets, int64_t *nnz_out) {
    return no_throw([&] {
        return compress_impl<uint8_t>(dense, rows, cols, bitmap, values, values_capacity, row_offsets, nnz_out);
    });
}

// The tile offset table of a bitmap, built on the host in exactly the layout the device
// kernels read (see endor_layout.h): the counter k of Algorithm 2 sampled every 4096
// positions, stored per 256-tile chunk.
extern "C" endor_status endor_build_offsets_host(int64_t rows, int64_t cols, const uint8_t *bitmap,
                                                 void *workspace, size_t workspace_bytes) {
    return no_throw([&]() -> endor_status {
    using namespace endor_layout;
    if (rows < 0 || cols < 0) return ENDOR_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols)) return ENDOR_ERR_UNSUPPORTED;
    const int64_t n = rows * cols;
    if (n == 0) return ENDOR_OK;
    if (!bitmap || !workspace) return ENDOR_ERR_INVALID_ARG;
    if (workspace_bytes < workspace_bytes_n(n)) return ENDOR_ERR_BUFFER_TOO_SMALL;
    const uint32_t nchunks = chunks_of(n);
    std::memset(workspace, 0, workspace_bytes_n(n));
    uint32_t *chunk_total = static_cast<uint32_t *>(workspace);
    uint32_t *tile_off = reinterpret_cast<uint32_t *>(static_cast<char *>(workspace) + chunk_total_bytes(n));
    const int64_t full_words = n / 64;
    const int tail_bits = static_cast<int>(n % 64);
    unsigned hw = std::thread::hardware_concurrency();
    const int nthreads = static_cast<int>(std::min<int64_t>(std::min<unsigned>(hw ? hw : 1, 64), nchunks));
    run_threads(nthreads, [&](int t) {
        for (uint32_t c = nchunks * uint64_t(t) / nthreads; c < nchunks * uint64_t(t + 1) / nthreads; ++c) {
            uint32_t run = 0;
            uint32_t *to = tile_off + size_t(c) * kChunkStride;
            for (int tl = 0; tl < kTilesPerChunk; ++tl) {
                to[tl] = run;
                const int64_t w0 = (int64_t(c) * kTilesPerChunk + tl) * kTileWords;
                for (int64_t w = w0; w < w0 + kTileWords; ++w) {
                    uint64_t m = 0;
                    if (w < full_words) {
                        std::memcpy(&m, bitmap + 8 * w, 8);
                    } else if (w == full_words && tail_bits) {
                        std::memcpy(&m, bitmap + 8 * w, 8);
                        m &= (uint64_t(1) << tail_bits) - 1;  // pad bits are ignored
                    }
                    run += static_cast<uint32_t>(__builtin_popcountll(m));
                }
            }
            to[kTilesPerChunk] = run;
            chunk_total[c] = run;
        }
    });
    return ENDOR_OK;
    });
}


// ---------------------------------------------------------------- row blocks for the pipeline

extern "C" endor_status endor_row_block_cuts(int64_t rows, int64_t cols, int nblocks, int64_t *cuts) {
    if (rows < 0 || cols < 0 || nblocks < 1 || !cuts) return ENDOR_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols)) return ENDOR_ERR_UNSUPPORTED;
    // smallest number of rows whose bits fill whole 64-bit words: 64 / gcd(cols, 64)
    const int64_t step = cols > 0 ? 64 / std::gcd<int64_t>(cols, 64) : 1;
    cuts[0] = 0;
    for (int b = 1; b < nblocks; ++b) {
        // rows*b < 2^34 * 2^31 fits 64 bits
        const int64_t r = rows * b / nblocks / step * step;
        cuts[b] = r < cuts[b - 1] ? cuts[b - 1] : r;
    }
    cuts[nblocks] = rows;
    return ENDOR_OK;
}

extern "C" endor_status endor_row_block(int64_t rows, int64_t cols, int elem_bytes, const uint8_t *h_bitmap,
                                        const void *h_values, const int64_t *row_offsets, int64_t r0, int64_t r1,
                                        void *d_dense, endor_host_blob *out) {
    if (!out || !row_offsets || rows < 0 || cols < 0 || (elem_bytes != 1 && elem_bytes != 2))
        return ENDOR_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols)) return ENDOR_ERR_UNSUPPORTED;
    if (r0 < 0 || r1 < r0 || r1 > rows) return ENDOR_ERR_INVALID_ARG;
    if ((r0 * cols) % 64 != 0) return ENDOR_ERR_INVALID_ARG;
    const int64_t k0 = row_offsets[r0], k1 = row_offsets[r1];
    if (k0 < 0 || k1 < k0) return ENDOR_ERR_INVALID_ARG;
    out->rows = r1 - r0;
    out->cols = cols;
    out->h_bitmap = h_bitmap ? h_bitmap + r0 * cols / 8 : nullptr;
    out->h_values = h_values ? static_cast<const char *>(h_values) + k0 * elem_bytes : nullptr;
    out->nnz = k1 - k0;
    out->d_dense = d_dense ? static_cast<char *>(d_dense) + r0 * cols * elem_bytes : nullptr;
    out->elem_bytes = elem_bytes;
    out->reserved = 0;
    return ENDOR_OK;
}
