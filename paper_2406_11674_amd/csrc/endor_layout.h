// Layout of the tile offset table inside a workspace, shared by the device kernels
// (endor_kernels.hip) and the host-side builder (endor_host.cpp).
//
// A matrix of n = rows*cols elements has ceil(n / 4096) tiles and ceil(tiles / 256)
// chunks.  Its workspace slice is
//     uint32 chunk_total[nchunks]            number of 1 bits in each chunk
//     (padding to a multiple of 256 bytes)
//     uint32 tile_off[nchunks][257]          1 bits before each tile, relative to the chunk
//                                            start; entry 256 repeats the chunk total
//     (padding to a multiple of 256 bytes)
// Tiles past the end of the matrix count as empty.
#ifndef ENDOR_LAYOUT_H_
#define ENDOR_LAYOUT_H_

#include <cstddef>
#include <cstdint>

#include "endor.h"

namespace endor_layout {

constexpr int kTileElems = ENDOR_TILE_ELEMS;
constexpr int kTileWords = kTileElems / 64;
constexpr int kTilesPerChunk = 256;  // chunk sizes of 64, 128 and 512 tiles measured no faster
constexpr int kChunkStride = kTilesPerChunk + 1;
constexpr int64_t kMaxElems = int64_t(1) << 34;

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

inline bool dims_ok(int64_t rows, int64_t cols) {
    if (rows < 0 || cols < 0) return false;
    if (rows == 0 || cols == 0) return true;
    return cols <= (kMaxElems - 1) / rows;  // rows*cols < 2^34, without overflow
}

inline uint32_t chunks_of(int64_t n) {
    const int64_t ntiles = (n + kTileElems - 1) / kTileElems;
    return static_cast<uint32_t>((ntiles + kTilesPerChunk - 1) / kTilesPerChunk);
}

inline size_t chunk_total_bytes(int64_t n) { return align256(size_t(chunks_of(n)) * sizeof(uint32_t)); }

inline size_t workspace_bytes_n(int64_t n) {
    return chunk_total_bytes(n) + align256(size_t(chunks_of(n)) * kChunkStride * sizeof(uint32_t));
}

}  // namespace endor_layout

#endif  // ENDOR_LAYOUT_H_
