// Host-side self-check run under AddressSanitizer + UBSan: endor_compress (several
// threads) against the plain oracle on ragged shapes, exact buffer sizes, so that any
// out-of-bounds access of the compressor is caught.  Built and run by
// tests/test_host_sanitizers.py; not part of the library.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "endor.h"

extern "C" {
int64_t oracle_compress(const void *dense, int elem_bytes, int64_t rows, int64_t cols, uint8_t *bitmap,
                        void *values, int64_t *row_offsets);
int64_t oracle_decompress(int elem_bytes, int64_t rows, int64_t cols, const uint8_t *bitmap, const void *values,
                          void *out);
}

static uint64_t state = 0x243F6A8885A308D3ull;
static uint64_t rnd() {
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return state;
}

template <class T>
static int check(int64_t rows, int64_t cols, int keep_of_256) {
    const int64_t n = rows * cols;
    std::vector<T> dense(n);
    for (auto &d : dense) {
        T v = static_cast<T>(rnd() | 1);
        d = (static_cast<int>(rnd() & 255) < keep_of_256) ? v : T(0);
    }
    std::vector<uint8_t> bitmap(endor_bitmap_bytes(rows, cols));
    std::vector<int64_t> ro(rows + 1);
    int64_t nnz = -1;
    endor_status st;
    if (sizeof(T) == 2)
        st = endor_compress(reinterpret_cast<const uint16_t *>(dense.data()), rows, cols, bitmap.data(), nullptr, 0,
                            ro.data(), &nnz);
    else
        st = endor_compress_u8(reinterpret_cast<const uint8_t *>(dense.data()), rows, cols, bitmap.data(), nullptr, 0,
                               ro.data(), &nnz);
    if (st != ENDOR_OK) return 1;
    std::vector<T> values(nnz);  // exactly nnz elements: one too many written would trip ASan
    if (sizeof(T) == 2)
        st = endor_compress(reinterpret_cast<const uint16_t *>(dense.data()), rows, cols, bitmap.data(),
                            reinterpret_cast<uint16_t *>(values.data()), nnz, ro.data(), &nnz);
    else
        st = endor_compress_u8(reinterpret_cast<const uint8_t *>(dense.data()), rows, cols, bitmap.data(),
                               reinterpret_cast<uint8_t *>(values.data()), nnz, ro.data(), &nnz);
    if (st != ENDOR_OK) return 2;
    // oracle side: Algorithm 1 gives the same streams, Algorithm 2 brings the matrix back
    std::vector<uint8_t> ob((n + 7) / 8 + 8);
    std::vector<T> ov(n ? n : 1);
    std::vector<int64_t> oro(rows + 1);
    const int64_t onnz = oracle_compress(dense.data(), sizeof(T), rows, cols, ob.data(), ov.data(), oro.data());
    if (onnz != nnz) return 3;
    if (n && std::memcmp(ob.data(), bitmap.data(), (n + 7) / 8) != 0) return 4;
    if (nnz && std::memcmp(ov.data(), values.data(), nnz * sizeof(T)) != 0) return 5;
    if (std::memcmp(oro.data(), ro.data(), (rows + 1) * sizeof(int64_t)) != 0) return 6;
    std::vector<T> back(n ? n : 1);
    oracle_decompress(sizeof(T), rows, cols, bitmap.data(), values.data(), back.data());
    if (n && std::memcmp(back.data(), dense.data(), n * sizeof(T)) != 0) return 7;
    return 0;
}

int main() {
    const int64_t shapes[][2] = {{1, 1}, {1, 63}, {1, 64}, {1, 65}, {3, 5}, {7, 13}, {129, 257}, {5, 4097},
                                 {0, 9}, {9, 0}, {1531, 4099}, {2048, 1024}};
    int cases = 0;
    for (auto &s : shapes)
        for (int keep : {0, 26, 128, 256}) {
            int rc = check<uint16_t>(s[0], s[1], keep);
            if (rc) { std::printf("fp16 %ldx%ld keep %d: failure %d\n", (long)s[0], (long)s[1], keep, rc); return 1; }
            rc = check<uint8_t>(s[0], s[1], keep);
            if (rc) { std::printf("u8 %ldx%ld keep %d: failure %d\n", (long)s[0], (long)s[1], keep, rc); return 1; }
            cases += 2;
        }
    std::printf("ok %d cases\n", cases);
    return 0;
}
