// Device side of the Endor library for gfx950 (MI355X): the parallel form of
// Algorithm 2 (Section 4.1, "Decompression") and the offset table it needs.
//
// Algorithm 2 is a sequential walk with one running counter k: position e of the
// flat bit vector receives values[k] when bit e is 1 (then k advances) and the
// all-zero pattern otherwise.  Hence out[e] = bit(e) ? values[rank(e)] : 0 with
// rank(e) = number of 1 bits before e, and the work splits into
//
//   1. endor_tile_offsets_kernel: rank at every tile start (a tile is 4096
//      consecutive flat positions = 64 bitmap words = one 64-lane wave's worth of
//      words).  One workgroup covers a chunk of 256 tiles: it popcounts the chunk's
//      128 KiB of bitmap, scans the 256 tile counts and stores the tile offsets
//      relative to the chunk start plus the chunk's total.
//   2. endor_expand_kernel: one single-wave workgroup per tile, waves fully
//      independent (no workgroup barrier; measured faster on MI355X than wider
//      workgroups or several tiles per wave).  The wave adds up the totals of the
//      chunks before its own (a few loads per lane) to get the chunk's absolute
//      start, brings the tile's contiguous slice of `values` straight from memory
//      into LDS (16 bytes per lane and load), scans the 64 word popcounts across
//      lanes (DPP), and then, in 8 steps
//      of 512 elements, every lane turns one bitmap byte into 8 output elements
//      (8 LDS reads at rank-within-byte offsets, masked by the bits) and issues one
//      16-byte store, so a wave writes 1 KiB of contiguous dense output per store
//      instruction.
//
// The same tile expander, fed differently, gives the row-subset kernel (Section 4.2's
// selective load) and - run backwards, as a scatter - the pack step of the device-side
// compressor (Algorithm 1).  The element width (2 bytes, or 1 for the 8-bit variant of
// Section 4.2) is a template parameter throughout.  The products on the compressed form
// (here the matrix-vector one; the small-batch one has a file of its own) expand in
// registers instead: a bitmap byte's values are one 16-byte window of `values`, read
// straight from memory and put in place with byte permutes.
//
// One rule shaped all of these kernels: a load under a per-lane test whose result is used
// after the test is waited for on the spot, so several of them in a row are as many trips
// to memory.  Loads are therefore either unconditional (behind one wave-uniform test, or
// from a clamped index, with the exceptional tiles in a loop of their own) or go straight
// to LDS.
//
// The path is bound by memory traffic (2 bytes written, 1/8 + 2p bytes read per
// element), so there is no matrix-core work here; all arithmetic on the format is
// integer and the values are only ever moved, never interpreted (the product kernel
// apart).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>

#include "endor.h"
#include "endor_device.h"
#include "endor_layout.h"

namespace {

using endor_device::chunk_base;
using endor_device::dpp_or_zero;
using endor_device::global_ptr;
using endor_device::global_ptr_mut;
using endor_device::load_to_lds16;
using endor_device::window_finish;
using endor_device::window_guarded;
using endor_device::window_issue;
using endor_device::WindowLoad;
using endor_device::windows_inside;
using endor_device::place_window;
using endor_device::window_tables_init;
using endor_device::WindowTables;
using endor_device::row_inclusive_scan;
using endor_device::u32x4;
using endor_device::wave_inclusive_scan;
using endor_device::wait_loads_to_lds;
using endor_device::wave_sum;

using endor_layout::kTileElems;      // flat positions per tile
using endor_layout::kTileWords;      // 64-bit bitmap words per tile (= lanes per wave)
using endor_layout::kTilesPerChunk;  // tiles one count workgroup covers
using endor_layout::kChunkStride;
using endor_layout::kMaxElems;
using endor_layout::align256;
using endor_layout::chunks_of;
using endor_layout::dims_ok;
using endor_layout::workspace_bytes_n;
constexpr int kBlock = 256;                   // threads per workgroup of the row-offset and column kernels
constexpr int kWaves = kBlock / 64;
// Launch shapes.  Both were settled by measurement on MI355X (Llama2-70B layer, half the
// elements kept): the tile-offset kernel with 16 waves per 256-tile chunk, the expand kernel
// with one single-wave workgroup per tile (wider workgroups, several tiles per wave and half
// tiles per wave were all slower), non-temporal value loads and stores, cacheable bitmap loads.
constexpr int kCountWaves = 16;               // waves per workgroup of the tile-offset kernel
constexpr int kCountBlock = 64 * kCountWaves;
constexpr int kCountTilesPerWave = kTilesPerChunk / kCountWaves;
constexpr int kCountSteps = kCountTilesPerWave / 2;  // two tiles per step

static_assert(kTileWords == 64, "one bitmap word per lane");
static_assert(kTilesPerChunk == 256 && kCountBlock >= kTilesPerChunk && kCountTilesPerWave % 2 == 0 &&
                  kCountSteps >= 1,
              "the tile-offset workgroup scans one tile count per thread");

struct MatParams {
    const uint64_t *bitmap;
    const void *values;     // nnz elements of 1 or 2 bytes
    void *dense;            // rows*cols elements of the same width
    uint32_t *chunk_total;  // [nchunks] 1 bits per chunk
    uint32_t *tile_off;     // [nchunks][257] 1 bits before each tile, relative to the chunk start
    int64_t n;              // rows*cols
    int64_t nnz;
    uint32_t chunk_begin;   // first workgroup-chunk of this matrix inside the batch
    uint32_t nchunks;
};

struct BatchParams {
    MatParams m[ENDOR_MAX_BATCH];
    // the matrices' chunk_begin again, side by side: a wave finds its matrix from one scalar load
    // of these instead of walking the descriptors (entries past `count` hold 0xffffffff)
    uint32_t first_chunk[ENDOR_MAX_BATCH];
    int count;
};

// Bitmap word `w` of a matrix with `full_words` complete words and `tail_bits`
// valid bits in the word after them; pad bits and words past the end read as 0.
__device__ __forceinline__ uint64_t load_word_guarded(const uint64_t *bitmap, int64_t w,
                                                      int64_t full_words, uint32_t tail_bits) {
    if (w < full_words) return bitmap[w];
    if (w == full_words && tail_bits != 0) return bitmap[w] & ((uint64_t(1) << tail_bits) - 1);
    return 0;
}

__device__ __forceinline__ int find_matrix(const BatchParams &P, uint32_t chunk) {
    int mi = 0;
#pragma unroll
    for (int i = 1; i < ENDOR_MAX_BATCH; ++i) mi += (chunk >= P.first_chunk[i]) ? 1 : 0;  // ascending, so a count
    return mi;
}

// ---------------------------------------------------------------- kernel 1: tile offsets

struct alignas(16) WordPair {
    uint64_t a, b;
};

// Workgroup of kCountWaves waves per chunk; wave w popcounts tiles
// [w*kCountTilesPerWave, (w+1)*kCountTilesPerWave) of the chunk in steps of two tiles
// (128 words: lanes 0..31 hold tile 2i, lanes 32..63 tile 2i+1, two words per lane),
// with all of its loads issued before the first popcount.
__global__ __launch_bounds__(kCountBlock) void endor_tile_offsets_kernel(BatchParams P) {
    __shared__ uint32_t s_cnt[kTilesPerChunk];
    __shared__ uint32_t s_wave[kTilesPerChunk / 64];

    const uint32_t gc = blockIdx.x;
    const MatParams &M = P.m[find_matrix(P, gc)];
    const uint32_t c = gc - M.chunk_begin;
    const uint64_t *bitmap = M.bitmap;
    const int64_t full_words = M.n >> 6;
    const uint32_t tail_bits = static_cast<uint32_t>(M.n & 63);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;

    const uint32_t t0 = wave * kCountTilesPerWave;  // first tile of this wave inside the chunk
    const int64_t wbase = (int64_t(c) * kTilesPerChunk + t0) * kTileWords;
    const bool all_fast = (reinterpret_cast<uintptr_t>(bitmap) & 15) == 0 &&
                          wbase + kCountSteps * 128 <= full_words;  // wave-uniform

    uint32_t p[kCountSteps];
    if (all_fast) {
        WordPair wp[kCountSteps];
#pragma unroll
        for (int i = 0; i < kCountSteps; ++i)
            wp[i] = *reinterpret_cast<const WordPair *>(bitmap + wbase + i * 128 + lane * 2);
#pragma unroll
        for (int i = 0; i < kCountSteps; ++i) p[i] = __popcll(wp[i].a) + __popcll(wp[i].b);
    } else {
#pragma unroll
        for (int i = 0; i < kCountSteps; ++i) {
            const int64_t w = wbase + i * 128 + lane * 2;
            p[i] = __popcll(load_word_guarded(bitmap, w, full_words, tail_bits)) +
                   __popcll(load_word_guarded(bitmap, w + 1, full_words, tail_bits));
        }
    }
#pragma unroll
    for (int i = 0; i < kCountSteps; ++i) {
        uint32_t q = row_inclusive_scan(p[i]);
        q += dpp_or_zero<0x142, 0xa>(q);  // lanes 31 and 63 now hold the two tile counts
        if ((lane & 31) == 31) s_cnt[t0 + 2 * i + (lane >> 5)] = q;
    }
    __syncthreads();

    if (threadIdx.x < kTilesPerChunk) {  // the first four waves scan the 256 tile counts
        const uint32_t cnt = s_cnt[threadIdx.x];
        const uint32_t incl = wave_inclusive_scan(cnt);
        if (lane == 63) s_wave[wave] = incl;
        s_cnt[threadIdx.x] = incl - cnt;
    }
    __syncthreads();
    if (threadIdx.x < kTilesPerChunk) {
        uint32_t before = 0;
        for (uint32_t v = 0; v < wave; ++v) before += s_wave[v];
        const uint32_t excl = before + s_cnt[threadIdx.x];
        uint32_t *to = M.tile_off + size_t(c) * kChunkStride;
        to[threadIdx.x] = excl;
        if (threadIdx.x == kTilesPerChunk - 1) {
            const uint32_t total = before + s_wave[wave];
            to[kTilesPerChunk] = total;
            M.chunk_total[c] = total;
        }
    }
}

// ---------------------------------------------------------------- kernel 2: expand

// Element width E in bytes: 2 (fp16, the paper's main case) or 1 (the 8-bit variant of
// Section 4.2).  A lane produces 16 bytes of output per step, i.e. kLaneElems elements
// covering kLaneElems bitmap bits; a tile of 4096 elements takes kSteps steps.
template <int E>
struct Shape {
    static constexpr int kLaneElems = 16 / E;                  // 8 or 16
    static constexpr int kSteps = kTileElems / (64 * kLaneElems);  // 8 or 4
    static constexpr int kLanesPerWord = 64 / kLaneElems;      // 8 or 4
};

// LDS a wave needs to expand a tile.  kCap = values the staging area holds at once: 4096 (a
// whole tile, whatever its density) or, for matrices known to be sparse, 1024 - a tile with more
// 1 bits than that is then expanded step by step (slower, but such tiles are rare there) and
// the smaller footprint lets more waves share a compute unit, which is what a store-dominated
// matrix wants (measured at one element in ten kept: 103 -> 97 us on 8192 x 28672).
template <int E, int kCap = kTileElems>
struct alignas(16) WaveScratch {
    static_assert(kCap >= 1024 && kCap <= kTileElems, "a step covers up to 1024 values");
    static constexpr int kLaneElems = Shape<E>::kLaneElems;
    // staging in 16-byte units: up to kLaneElems-1 elements of alignment slack in front, kCap
    // values, and kLaneElems-1 elements a lane may read past its last value (those reads are
    // masked off by the bits)
    // (8-bit values are read as dword pairs around a lane's values, up to 4 bytes further: one unit more)
    static constexpr int kStageChunks = (E * (2 * (kLaneElems - 1) + kCap) + 15) / 16 + (E == 1 ? 1 : 0);
    static constexpr int kStageRounds = (kStageChunks + 63) / 64;
    // last index a lane's values may start at
    static constexpr uint32_t kMaxIndex = (kStageChunks - (E == 1 ? 1 : 0)) * (16 / E) - kLaneElems;
    u32x4 stage[kStageChunks];   // the tile's slice of `values`, from the 16-byte boundary below it
    uint64_t words[kTileWords];  // the tile's bitmap words
    uint32_t start[kTileWords];  // per word: index into `stage` (in elements) of its first value
    // 8-bit values only: per 4-bit pattern the v_perm_b32 selector that moves the pattern's
    // consecutive values to the positions of its 1 bits and zeroes the others
    uint32_t nibble_sel[E == 1 ? 16 : 1];
};

// Selector for pattern n (bits 0..3): output byte k takes source byte popcount(n below k) when
// bit k is set, and the constant zero (selector 0x0c) otherwise.
__device__ __forceinline__ uint32_t nibble_selector(uint32_t n) {
    uint32_t sel = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k)
        sel |= (((n >> k) & 1u) ? uint32_t(__popc(n & ((1u << k) - 1))) : 0x0cu) << (8 * k);
    return sel;
}

// 16 bytes of `values` at byte address p, with bytes outside [vbeg, vend) read as 0
template <int E>
__device__ __forceinline__ u32x4 load_values16(uintptr_t p, uintptr_t vbeg, uintptr_t vend) {
    // values are read once: streamed past the caches (the bitmap, read by both kernels, stays cacheable)
    if (p >= vbeg && p + 16 <= vend) return __builtin_nontemporal_load(global_ptr<u32x4>(p));
    uint32_t d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 16 / E; ++j) {
        const uintptr_t q = p + E * j;
        uint32_t v = 0;
        if (q >= vbeg && q + E <= vend)
            v = (E == 2) ? uint32_t(*global_ptr<uint16_t>(q)) : uint32_t(*global_ptr<uint8_t>(q));
        d[(E * j) >> 2] |= v << (8 * ((E * j) & 3));
    }
    u32x4 r;
    r.x = d[0];
    r.y = d[1];
    r.z = d[2];
    r.w = d[3];
    return r;
}

// 0xffff in the halves whose bit is set: bits 0,1 of `b` -> low, high half
__device__ __forceinline__ uint32_t half_mask(uint32_t b) {
    return ((b & 1u) ? 0xffffu : 0u) | ((b & 2u) ? 0xffff0000u : 0u);
}

// Sink that writes the expanded tile to memory: a 16-byte non-temporal store per lane
// and step when the tile is complete and the output 16-byte aligned, else element by
// element with a bounds check.  kBurst holds the steps' results back and releases all of
// them after the last step: measured 11 % faster when almost everything is stores (one
// element in ten kept), 6 % slower at three in ten, so the host picks it by density.
template <int E, bool kAlignedOut, bool kBurst>
struct StoreSink {
    uint8_t *out;     // byte address of the tile's first output element
    uint32_t nvalid;  // elements of the tile that exist (<= 4096)
    u32x4 held[kBurst ? Shape<E>::kSteps : 1];
    // how far a loop over the steps must be unrolled for `held` to stay in registers
    static constexpr int kStepUnroll = kBurst ? Shape<E>::kSteps : 1;
    __device__ __forceinline__ void put(uint32_t le, u32x4 d) const {
        __builtin_nontemporal_store(d, reinterpret_cast<u32x4 *>(out + size_t(le) * E));
    }
    __device__ __forceinline__ void operator()(int k, uint32_t le, u32x4 d) {
        if (kAlignedOut && nvalid == kTileElems) {
            if (kBurst) {
                held[k] = d;
                if (k == Shape<E>::kSteps - 1) {
#pragma unroll
                    for (int g = 0; g < Shape<E>::kSteps; ++g)
                        put(le - (Shape<E>::kSteps - 1 - g) * 64 * Shape<E>::kLaneElems, held[g]);
                }
            } else {
                put(le, d);
            }
        } else {
            const uint32_t dd[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
            for (int j = 0; j < Shape<E>::kLaneElems; ++j) {
                if (le + j < nvalid) {
                    const uint32_t v = dd[(E * j) >> 2] >> (8 * ((E * j) & 3));
                    if (E == 2)
                        reinterpret_cast<uint16_t *>(out)[le + j] = static_cast<uint16_t>(v);
                    else
                        out[le + j] = static_cast<uint8_t>(v);
                }
            }
        }
    }
};

// One step of the expansion: every lane turns kLaneElems bitmap bits into 16 bytes of output.
// S.words and S.start (per word: index into S.stage of its first value) are in place.
template <int E, int kCap, class Sink>
__device__ __forceinline__ void expand_step(const WaveScratch<E, kCap> &S, int k, uint32_t lane, Sink &sink) {
    using Sh = Shape<E>;
    const uint32_t wi = k * Sh::kLaneElems + lane / Sh::kLanesPerWord;
    const uint64_t w = S.words[wi];
    const uint32_t sh = (lane % Sh::kLanesPerWord) * Sh::kLaneElems;
    const uint32_t bits = static_cast<uint32_t>(w >> sh) & ((1u << Sh::kLaneElems) - 1);
    uint32_t s = S.start[wi] + __popcll(w & ((uint64_t(1) << sh) - 1));
    // with a whole tile staged the index cannot leave the staging area; with a smaller area a
    // table that does not belong to the bitmap could make it, so it is clamped
    if (kCap < kTileElems) s = s > WaveScratch<E, kCap>::kMaxIndex ? WaveScratch<E, kCap>::kMaxIndex : s;
    // every element is read from the staging area at its rank; the ones whose bit is 0
    // pick up a neighbour's value and are masked to the all-zero pattern.
    u32x4 d;
    if (E == 2) {
        const uint16_t *sp = reinterpret_cast<const uint16_t *>(S.stage) + s;
        uint32_t h[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) h[j] = sp[__popc(bits & ((1u << j) - 1))];
        d.x = (h[0] | (h[1] << 16)) & half_mask(bits);
        d.y = (h[2] | (h[3] << 16)) & half_mask(bits >> 2);
        d.z = (h[4] | (h[5] << 16)) & half_mask(bits >> 4);
        d.w = (h[6] | (h[7] << 16)) & half_mask(bits >> 6);
    } else {
        // 8-bit values: an output dword's four elements take consecutive values, so one read of the
        // two dwords around them, a funnel shift and a byte permute replace four single-byte
        // gathers (the 8-bit kernel was bound by vector ALU and LDS instructions, not by memory)
        const uint32_t *sw = reinterpret_cast<const uint32_t *>(S.stage);
        uint32_t o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t at = s + __popc(bits & ((1u << (4 * q)) - 1));  // byte index of the dword's first value
            const uint32_t lo = sw[at >> 2], hi = sw[(at >> 2) + 1];
            const uint32_t x = __builtin_amdgcn_alignbyte(hi, lo, at & 3u);
            o[q] = __builtin_amdgcn_perm(x, x, S.nibble_sel[(bits >> (4 * q)) & 15u]);
        }
        d.x = o[0];
        d.y = o[1];
        d.z = o[2];
        d.w = o[3];
    }
    sink(k, (k * 64 + lane) * Sh::kLaneElems, d);
}

// LDS operations of one wave execute in issue order, so reads after this point see the writes
// before it; the fences only keep the compiler from moving them.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Expand one tile with one wave.
//   word     this lane's 64 bitmap bits of the tile (bits past the end already cleared)
//   vaddr    byte address of the tile's first value; cnt = number of 1 bits in the tile
//   [vbeg, vend)  the byte range of the whole `values` array (nothing outside is read)
//   sink     receives, per step k, the 16 expanded bytes of this lane: sink(k, le, d) with le
//            the index inside the tile of the lane's first element
// The caller has not touched S since the wave's previous call returned.
// (Measured alternatives to the per-element gather that lost for the store-bound kernels: one
// 32-bit read per output dword plus a byte permutation, with misaligned reads 1.8x slower,
// with aligned pairs and a funnel shift 1.0-1.4x.)
template <int E, int kCap, class Sink>
__device__ __forceinline__ void expand_tile(WaveScratch<E, kCap> &S, uint32_t lane, uint64_t word, uintptr_t vaddr,
                                            uint32_t cnt, uintptr_t vbeg, uintptr_t vend, Sink &sink) {
    using Sh = Shape<E>;
    using WS = WaveScratch<E, kCap>;
    // --- the loads of the tile's value slice (16-byte units from the 16-byte boundary at or
    //     below its first value) go out first: they depend on the table only, and the wave's
    //     bitmap word, loaded by the caller, may still be on its way
    const uintptr_t a16 = vaddr & ~uintptr_t(15);
    const uint32_t shift = static_cast<uint32_t>(vaddr - a16) / E;  // elements of slack in front
    if (E == 1 && lane < 16) S.nibble_sel[lane] = nibble_selector(lane);
    cnt = cnt > kCap ? kCap : cnt;  // a stale or foreign table must not overrun the staging area
    const uint32_t nch = cnt ? (((shift + cnt) * E + 15) >> 4) : 0;  // < kStageChunks
    // the whole slice lies inside `values`: all tiles but the first and last of an array that
    // does not begin and end on 16-byte boundaries
    const bool direct = nch != 0 && a16 >= vbeg && a16 + 16 * uintptr_t(nch) <= vend;
    if (direct) {
        // Straight from memory into the staging area (global_load_lds_dwordx4: lane l of an
        // instruction deposits its 16 bytes at the LDS address in M0 plus 16*l), no registers
        // in between.  Values are read once: streamed past the caches.
#pragma unroll
        for (int q = 0; q < WS::kStageRounds; ++q) {
            const uint32_t ch = q * 64 + lane;
            if (ch < nch) load_to_lds16(reinterpret_cast<const u32x4 *>(a16) + ch, &S.stage[q * 64]);
        }
    }
    const uint32_t pc = __popcll(word);
    const uint32_t incl = wave_inclusive_scan(pc);
    const uint32_t excl = incl - pc;
    if (kCap < kTileElems) {
        // more 1 bits than the staging area holds (decided on the bitmap itself, not on the
        // table): stage and expand the tile one step at a time; a step has at most 1024 values
        const uint32_t ones = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(incl), 63));
        if (ones > kCap) {  // wave-uniform
            if (direct) wait_loads_to_lds();  // what is on its way into the staging area lands before it is reused
            S.words[lane] = word;
#pragma unroll Sink::kStepUnroll
            for (int k = 0; k < Sh::kSteps; ++k) {
                // values before the step's first word; the step's own count
                const uint32_t w0 = k * Sh::kLaneElems;
                const uint32_t first = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(4 * w0, static_cast<int>(excl)));
                const uint32_t last = static_cast<uint32_t>(
                    __builtin_amdgcn_ds_bpermute(4 * (w0 + Sh::kLaneElems - 1), static_cast<int>(incl)));
                const uintptr_t va = vaddr + uintptr_t(E) * first;
                const uintptr_t b16 = va & ~uintptr_t(15);
                const uint32_t sh = static_cast<uint32_t>(va - b16) / E;
                const uint32_t n = last - first;  // <= 1024 <= kCap
                const uint32_t nc = n ? (((sh + n) * E + 15) >> 4) : 0;
                S.start[lane] = excl - first + sh;  // meaningful for the step's words only
                for (uint32_t ch = lane; ch < nc; ch += 64)
                    S.stage[ch] = load_values16<E>(b16 + 16 * uintptr_t(ch), vbeg, vend);
                wave_lds_sync();
                expand_step<E, kCap>(S, k, lane, sink);
                wave_lds_sync();
            }
            return;
        }
    }
    S.words[lane] = word;
    S.start[lane] = excl + shift;
    if (direct) {
        wait_loads_to_lds();
    } else {
#pragma unroll 1
        for (uint32_t ch = lane; ch < nch; ch += 64)
            S.stage[ch] = load_values16<E>(a16 + 16 * uintptr_t(ch), vbeg, vend);
    }
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < Sh::kSteps; ++k) expand_step<E, kCap>(S, k, lane, sink);
    // the next tile's LDS writes must stay behind this tile's LDS reads
    wave_lds_sync();
}

// kCap: values the staging area holds (the host picks it from the batch's density); kBurst: all
// stores of a tile released together (for store-dominated matrices).
template <int E, bool kAlignedOut, int kCap, bool kBurst>
__global__ __launch_bounds__(64) void endor_expand_kernel(BatchParams P) {
    __shared__ WaveScratch<E, kCap> s_scratch;
    const uint32_t gc = blockIdx.x / kTilesPerChunk;
    const uint32_t tl = blockIdx.x % kTilesPerChunk;  // tile, relative to the chunk
    const MatParams &M = P.m[find_matrix(P, gc)];
    const uint32_t c = gc - M.chunk_begin;
    const uint32_t lane = threadIdx.x;

    const int64_t n = M.n;
    const int64_t ntiles = (n + kTileElems - 1) / kTileElems;
    const int64_t tile = int64_t(c) * kTilesPerChunk + tl;
    if (tile >= ntiles) return;

    const int64_t full_words = n >> 6;
    const uint32_t tail_bits = static_cast<uint32_t>(n & 63);
    const uintptr_t vbeg = reinterpret_cast<uintptr_t>(M.values);
    const uintptr_t vend = vbeg + E * static_cast<uintptr_t>(M.nnz);
    // the bitmap word first: its load is in flight while the table is looked up
    const uint64_t word = load_word_guarded(M.bitmap, tile * kTileWords + lane, full_words, tail_bits);
    const uint32_t *tile_off = M.tile_off + size_t(c) * kChunkStride + tl;
    const uint32_t o0 = tile_off[0];
    const uint32_t o1 = tile_off[1];
    const uint64_t base = chunk_base(M.chunk_total, c, lane);
    const uint32_t cnt = o1 - o0;  // 1 bits in this tile
    const int64_t e0 = tile * kTileElems;
    const int64_t left = n - e0;
    StoreSink<E, kAlignedOut, kBurst> sink;
    sink.out = reinterpret_cast<uint8_t *>(M.dense) + e0 * E;
    sink.nvalid = left < kTileElems ? static_cast<uint32_t>(left) : uint32_t(kTileElems);
    expand_tile<E>(s_scratch, lane, word, vbeg + E * (base + o0), cnt, vbeg, vend, sink);
}

// This lane's 64 bits of a segment of `nbits` (<= 4096) bits that starts at an arbitrary
// bit position e of the bitmap: bits e + 64*lane .. +63, funnelled out of two neighbouring
// words, with everything past the segment (or past the bitmap) cleared.
__device__ __forceinline__ uint64_t segment_word(const uint64_t *bitmap, int64_t nwords, int64_t e,
                                                 uint32_t nbits, uint32_t lane) {
    // Both loads are unconditional, from indices clamped into the bitmap, and the cases are
    // sorted out with selects afterwards: under a test each load would be waited for on the
    // spot, and a caller that fetches the next segment's word ahead would gain nothing.
    const int64_t w0 = (e >> 6) + lane;
    const uint32_t bs = static_cast<uint32_t>(e & 63);
    const int64_t last = nwords - 1;  // nwords >= 1: the callers have at least one element
    const uint64_t lo = bitmap[w0 < last ? w0 : last];
    const uint64_t hi = bitmap[w0 + 1 < last ? w0 + 1 : last];
    uint64_t word = (w0 < nwords ? lo : 0) >> bs;
    word |= ((w0 + 1 < nwords ? hi : 0) << 1) << (63 - bs);  // hi << (64 - bs), and nothing when bs is 0
    const uint32_t have = lane * 64 < nbits ? nbits - lane * 64 : 0u;  // bits of this lane that belong to the segment
    if (have < 64) word &= (uint64_t(1) << have) - 1;
    return word;
}

// ---------------------------------------------------------------- kernel 2b: selected rows

struct RowsParams {
    const uint64_t *bitmap;
    const void *values;
    void *out;                   // nsel x cols
    const int64_t *row_offsets;  // rows + 1
    const int64_t *sel;          // nsel row indices
    int64_t rows, cols, nnz, nsel;
    uint32_t segs;               // ceil(cols / 4096) tiles per row
};

// Row-subset decompression (the selective load of Section 4.2): output row r is row
// sel[r] of the matrix.  One wave per (selected row, 4096-column segment).  The segment
// starts at an arbitrary bit position, so a lane's 64 bits are funnelled out of two
// neighbouring bitmap words; its first value is row_offsets[row] plus the 1 bits of the
// row's earlier segments, counted here from the bitmap.
template <int E, bool kAlignedOut, int kCap = kTileElems>
__global__ __launch_bounds__(64) void endor_expand_rows_kernel(RowsParams R) {
    __shared__ WaveScratch<E, kCap> s_scratch;
    const uint32_t lane = threadIdx.x;
    const int64_t r = blockIdx.x / R.segs;
    const uint32_t g = blockIdx.x % R.segs;
    const int64_t i = R.sel[r];
    if (i < 0 || i >= R.rows) return;  // an index outside the matrix leaves its output row untouched

    const int64_t n = R.rows * R.cols;
    const int64_t nwords = (n + 63) >> 6;
    const int64_t row_bit = i * R.cols;                  // first bit of the row
    const int64_t e = row_bit + int64_t(g) * kTileElems;  // first bit of the segment
    const int64_t left = R.cols - int64_t(g) * kTileElems;
    const uint32_t nbits = left < kTileElems ? static_cast<uint32_t>(left) : uint32_t(kTileElems);

    // everything that depends on the row index only goes out together: the segment's own bits,
    // the row's first value, and the bitmap words before the segment
    const uint64_t word = segment_word(R.bitmap, nwords, e, nbits, lane);
    const uint64_t row_first = static_cast<uint64_t>(R.row_offsets[i]);

    // 1 bits of the row before this segment: words [row_bit>>6, e>>6], first and last partial.
    // A lane's share stays below 2^28; the total may not fit 32 bits for very wide rows, so
    // the two 16-bit halves are summed across the wave separately.  Two words per lane and
    // pass, loaded unconditionally (an index past the last word reads the last again and is
    // dropped), so that a pass is one trip to memory.
    uint64_t before = 0;
    {
        uint32_t part = 0;
        const int64_t wa = row_bit >> 6, wb = e >> 6;  // wb < nwords: e is a position of the matrix
        for (int64_t w0 = wa; w0 <= wb; w0 += 128) {
            uint64_t x[2];
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int64_t w = w0 + 64 * k + lane;
                x[k] = R.bitmap[w <= wb ? w : wb];
            }
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int64_t w = w0 + 64 * k + lane;
                uint64_t y = w <= wb ? x[k] : 0;
                if (w == wa) y &= ~uint64_t(0) << (row_bit & 63);
                if (w == wb) y &= (uint64_t(1) << (e & 63)) - 1;
                part += __popcll(y);
            }
        }
        before = uint64_t(wave_sum(part & 0xffffu)) + (uint64_t(wave_sum(part >> 16)) << 16);
    }
    const uint32_t cnt = wave_sum(__popcll(word));

    const uintptr_t vbeg = reinterpret_cast<uintptr_t>(R.values);
    const uintptr_t vend = vbeg + E * static_cast<uintptr_t>(R.nnz);
    const uint64_t first = row_first + before;
    StoreSink<E, kAlignedOut, false> sink;
    sink.out = reinterpret_cast<uint8_t *>(R.out) + (r * R.cols + int64_t(g) * kTileElems) * E;
    sink.nvalid = nbits;
    expand_tile<E, kCap>(s_scratch, lane, word, vbeg + E * first, cnt, vbeg, vend, sink);
}

// ---------------------------------------------------------------- kernel 2c: selected columns

struct ColsParams {
    const uint64_t *bitmap;
    const void *values;
    void *out;                   // rows x nsel
    const int64_t *row_offsets;  // rows + 1
    const int64_t *sel;          // nsel column indices
    int64_t rows, cols, nnz, nsel;
};

// 64 bits of row-aligned "virtual word" k of a row that starts at bit row_bit: bits
// row_bit + 64k .. +63, clipped to the row's `cols` bits and to the bitmap.
__device__ __forceinline__ uint64_t row_word(const uint64_t *bitmap, int64_t nwords, int64_t row_bit,
                                             int64_t cols, int64_t k) {
    const int64_t e = row_bit + 64 * k;
    const int64_t w0 = e >> 6;
    const uint32_t bs = static_cast<uint32_t>(e & 63);
    uint64_t word = (w0 < nwords ? bitmap[w0] : 0) >> bs;
    if (bs != 0) word |= (w0 + 1 < nwords ? bitmap[w0 + 1] : 0) << (64 - bs);
    const int64_t rem = cols - 64 * k;
    if (rem < 64) word &= (uint64_t(1) << rem) - 1;
    return word;
}

// Column-subset decompression (the other half of Section 4.2's selective load: the columns
// of a down projection that belong to active neurons).  out[i][q] = W[i][sel[q]].  One
// workgroup per row.  It first lays the row's bitmap out in LDS as 32-bit pieces, each with
// the number of the row's 1 bits before it; a query is then one coalesced load of its
// column index, two LDS reads and a handful of 32-bit operations for
//     rank = row_offsets[i] + before[piece] + popcount(bits of the piece below the column),
// and one 2-byte load of values[rank] (or a zero).  Queries are taken four at a time so that
// their loads are in flight together.  (Measured alternative that lost: streaming the row's
// whole value slice into LDS first and gathering from there - the 30-50 KB of LDS per row
// leave three workgroups per compute unit and the kernel becomes latency-bound: 110-150 us
// against 80 us for a tenth of the columns of 8192 x 28672.)
template <int E>
__global__ __launch_bounds__(kBlock) void endor_gather_cols_kernel(ColsParams C) {
    extern __shared__ uint32_t s_dyn[];  // [np] 32-bit pieces of the row's bitmap | [np] 1 bits of the row before each
    __shared__ uint32_t s_wave[2][kWaves];
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    const int64_t i = blockIdx.x;
    const int64_t nwords = (C.rows * C.cols + 63) >> 6;
    const int64_t row_bit = i * C.cols;
    const uint32_t nvw = static_cast<uint32_t>((C.cols + 63) >> 6);
    uint32_t *s_piece = s_dyn;
    uint32_t *s_before = s_dyn + 2 * nvw;

    // first round of column indices: in flight during the bitmap work
    constexpr int kQ = 4;  // queries per thread and round
    int64_t c[kQ];
#pragma unroll
    for (int u = 0; u < kQ; ++u) {
        const int64_t q = u * kBlock + threadIdx.x;
        c[u] = q < C.nsel ? C.sel[q] : -1;
    }

    // scan of the word popcounts, kBlock words per round: wave scan, then the waves' totals
    // through LDS (two alternating slots, so one barrier per round is enough)
    uint32_t carry = 0;
    for (uint32_t k0 = 0, round = 0; k0 < nvw; k0 += kBlock, ++round) {
        const uint32_t k = k0 + threadIdx.x;
        const uint64_t w = k < nvw ? row_word(C.bitmap, nwords, row_bit, C.cols, k) : 0;
        const uint32_t lo = static_cast<uint32_t>(w), hi = static_cast<uint32_t>(w >> 32);
        const uint32_t pc = __popc(lo) + __popc(hi);
        const uint32_t incl = wave_inclusive_scan(pc);
        if (lane == 63) s_wave[round & 1][wave] = incl;
        __syncthreads();
        uint32_t before = carry;
#pragma unroll
        for (uint32_t v = 0; v < kWaves; ++v) {
            const uint32_t t = s_wave[round & 1][v];
            before += v < wave ? t : 0;
            carry += t;
        }
        if (k < nvw) {
            const uint32_t excl = before + incl - pc;
            s_piece[2 * k] = lo;
            s_piece[2 * k + 1] = hi;
            s_before[2 * k] = excl;
            s_before[2 * k + 1] = excl + __popc(lo);
        }
    }
    __syncthreads();

    const int64_t row_first = C.row_offsets[i];
    // values from the row's first to the end of the array; none if the offset is not inside it
    const uint64_t room = (row_first >= 0 && row_first <= C.nnz) ? static_cast<uint64_t>(C.nnz - row_first) : 0;
    const uint8_t *row_values = static_cast<const uint8_t *>(C.values) + E * row_first;
    uint8_t *row_out = static_cast<uint8_t *>(C.out) + E * i * C.nsel;
    const uint64_t ucols = static_cast<uint64_t>(C.cols);
    for (int64_t q0 = 0; q0 < C.nsel; q0 += kQ * kBlock) {
        int64_t cn[kQ];
#pragma unroll
        for (int u = 0; u < kQ; ++u) {  // the next round's indices
            const int64_t q = q0 + (kQ + u) * kBlock + threadIdx.x;
            cn[u] = q < C.nsel ? C.sel[q] : -1;
        }
        uint32_t v[kQ];
        bool live[kQ], hit[kQ];
#pragma unroll
        for (int u = 0; u < kQ; ++u) {
            // an index outside the matrix (or past nsel) leaves its output column untouched
            live[u] = static_cast<uint64_t>(c[u]) < ucols;
            const uint32_t cc = live[u] ? static_cast<uint32_t>(c[u]) : 0u;
            const uint32_t piece = s_piece[cc >> 5];
            const uint32_t b = cc & 31;
            const uint32_t r = s_before[cc >> 5] + __popc(piece & ((1u << b) - 1));  // rank inside the row
            hit[u] = live[u] && ((piece >> b) & 1) != 0 && r < room;
            // The load itself is unconditional (a query without a value reads the first selected
            // index instead and drops it): with the load under the test, the compiler waits for
            // memory after every query and every store, one at a time.
            const uint8_t *at = hit[u] ? row_values + size_t(E) * r : reinterpret_cast<const uint8_t *>(C.sel);
            v[u] = (E == 2) ? uint32_t(*reinterpret_cast<const uint16_t *>(at)) : uint32_t(*at);
        }
#pragma unroll
        for (int u = 0; u < kQ; ++u) v[u] = hit[u] ? v[u] : 0u;
#pragma unroll
        for (int u = 0; u < kQ; ++u) {
            const int64_t q = q0 + u * kBlock + threadIdx.x;
            if (live[u]) {
                if (E == 2)
                    reinterpret_cast<uint16_t *>(row_out)[q] = static_cast<uint16_t>(v[u]);
                else
                    row_out[q] = static_cast<uint8_t>(v[u]);
            }
            c[u] = cn[u];
        }
    }
}

// ---------------------------------------------------------------- fused consumer: y = W x

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float wave_sum_f32(float x) {
    // same lane order as wave_inclusive_scan, so the result does not depend on timing
#define ENDOR_DPP_ADD_F32(ctrl, rowmask)                                                                     \
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), ctrl, rowmask, \
                                                               0xf, true))
    ENDOR_DPP_ADD_F32(0x111, 0xf);
    ENDOR_DPP_ADD_F32(0x112, 0xf);
    ENDOR_DPP_ADD_F32(0x114, 0xf);
    ENDOR_DPP_ADD_F32(0x118, 0xf);
    ENDOR_DPP_ADD_F32(0x142, 0xa);
    ENDOR_DPP_ADD_F32(0x143, 0xc);
#undef ENDOR_DPP_ADD_F32
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}

// Sink that multiplies the expanded fp16 elements with the matching 8 entries of x and
// accumulates in fp32.  Each product of two fp16 numbers is exact in fp32 and each step is
// one fused multiply-add with fp16 operands widened in the instruction (v_fma_mix_f32), so
// fp16 subnormals count in full (the packed dot-product instructions flush them).
struct GemvSink {
    float acc;
    __device__ __forceinline__ void pair(uint32_t w2, uint32_t x2) {
#pragma clang fp contract(off)  // keep the two multiply-adds apart: fused into a dot product they would flush
        const f16x2 w = __builtin_bit_cast(f16x2, w2);
        const f16x2 x = __builtin_bit_cast(f16x2, x2);
        acc = __builtin_fmaf(static_cast<float>(w.x), static_cast<float>(x.x), acc);
        acc = __builtin_fmaf(static_cast<float>(w.y), static_cast<float>(x.y), acc);
    }
    // 8 expanded elements against the matching 8 entries of x
    __device__ __forceinline__ void operator()(u32x4 d, u32x4 x) {
        pair(d.x, x.x);
        pair(d.y, x.y);
        pair(d.z, x.z);
        pair(d.w, x.w);
    }
};

struct GemvParams {
    const uint64_t *bitmap;
    const uint16_t *values;
    const int64_t *row_offsets;  // rows + 1
    const uint16_t *x;           // cols fp16
    float *y;                    // rows fp32
    int64_t rows, cols, nnz;
};

// y[i] = sum_j W[i][j] * x[j] straight from the compressed form: the dense row is never
// written.  One wave per row walks the row's 4096-column segments.  Per segment: popcount and
// scan the lane's bitmap word, leave one entry per bitmap byte in LDS ((values of the segment
// before the byte) << 8 | the byte); then a lane takes the bytes lane, 64 + lane, ... in turn,
// reads each byte's window of values straight from memory, places the values by the byte's
// bit pattern and feeds the fp16 pairs to multiply-adds against the matching 8 entries of x.
// Elements whose bit is 0 enter as +0.0, as they would from the dense matrix.  The next
// segment's bitmap word is loaded before the current one is worked on.
// (Measured alternatives on 28672 x 8192, half kept: values staged in LDS and gathered element
// by element 83 us, staged and read as windows 76 us, windows straight from memory 72 us, and
// with x shared through LDS as below 64-67 us; a wave taking four rows in turn 143 us: a wave's
// segments run one after the other, so what counts is the number of independent waves.  Counters
// of the 72 us form: the vector cache handles some 530 line accesses per segment, 128 of them
// for x, where 200 would do if no two lanes shared a line.)
constexpr int kGemvSeg = 4096;  // columns a wave expands at a time

// kFastX: x is 16-byte aligned and cols a multiple of 8, so x moves in whole aligned 16-byte
// pieces (the general path builds each piece from 8 guarded loads).
//
// The kGemvWaves rows of a workgroup walk their segments in step, so the segment's 4096 entries
// of x are brought to LDS once per workgroup (one 16-byte piece per thread, straight from
// memory into LDS on the fast path, double buffered, one barrier per segment) instead of once
// per row: x is the same 8 KB for every row, and fetching it per row cost a quarter of the
// vector cache's accesses.
constexpr int kGemvWaves = 8;
constexpr int kGemvXRounds = (kGemvSeg / 8 + 64 * kGemvWaves - 1) / (64 * kGemvWaves);  // 16-byte pieces of x per thread and segment

template <bool kFastX>
__global__ __launch_bounds__(64 * kGemvWaves) void endor_gemv_f16_kernel(GemvParams G) {
    __shared__ WindowTables s_tables;
    __shared__ uint32_t s_entry[kGemvWaves][kGemvSeg / 8];
    __shared__ u32x4 s_x[2][kGemvSeg / 8];
    window_tables_init(s_tables, threadIdx.x);  // visible after the first segment's barrier
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    const int64_t i = int64_t(blockIdx.x) * kGemvWaves + wave;
    const bool row_ok = i < G.rows;  // a wave past the last row still helps loading x
    uint32_t *entry = s_entry[wave];
    const int64_t nwords = (G.rows * G.cols + 63) >> 6;
    const int64_t row_bit = (row_ok ? i : 0) * G.cols;
    const uintptr_t vbeg = reinterpret_cast<uintptr_t>(G.values);
    const uintptr_t vend = vbeg + 2 * static_cast<uintptr_t>(G.nnz);
    uint64_t next_value = row_ok ? static_cast<uint64_t>(G.row_offsets[i]) : 0;
    GemvSink sink;
    sink.acc = 0.0f;

    // this thread's piece of the segment of x that starts at column c0
    auto load_x = [&](int64_t c0, uint32_t buf) {
#pragma unroll
        for (int q = 0; q < kGemvXRounds; ++q) {
            const uint32_t piece = q * 64 * kGemvWaves + threadIdx.x;
            if (64 * kGemvWaves * kGemvXRounds > kGemvSeg / 8 && piece >= kGemvSeg / 8) break;  // more threads than pieces
            const int64_t c = c0 + 8 * int64_t(piece);
            if (kFastX) {
                // past the row's end x reads as zero (the expanded elements there are zero, but
                // zero times whatever LDS held could be NaN)
                if (c < G.cols)
                    load_to_lds16<false>(reinterpret_cast<const u32x4 *>(G.x + c), &s_x[buf][q * 64 * kGemvWaves + 64 * wave]);
                else
                    s_x[buf][piece] = u32x4{0u, 0u, 0u, 0u};
            } else {
                uint32_t h[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) h[j] = (c + j < G.cols) ? uint32_t(G.x[c + j]) : 0u;
                u32x4 f;
                f.x = h[0] | (h[1] << 16);
                f.y = h[2] | (h[3] << 16);
                f.z = h[4] | (h[5] << 16);
                f.w = h[6] | (h[7] << 16);
                s_x[buf][piece] = f;
            }
        }
    };
    auto row_word = [&](int64_t c0) -> uint64_t {  // no branch: a segment that does not exist has no bits
        const int64_t left = G.cols - c0;
        const uint32_t nbits = (!row_ok || left <= 0) ? 0u : left < kGemvSeg ? static_cast<uint32_t>(left) : uint32_t(kGemvSeg);
        return segment_word(G.bitmap, nwords, row_bit + c0, nbits, lane);
    };

    if (G.cols > 0) load_x(0, 0);
    uint64_t word = row_word(0);
    uint32_t buf = 0;
    for (int64_t c0 = 0; c0 < G.cols; c0 += kGemvSeg, buf ^= 1u) {
        const int64_t left = G.cols - c0;
        // this thread's piece of the segment's x has landed; after the barrier all of them have,
        // and every wave is through the previous segment (whose x the next load overwrites)
        wait_loads_to_lds();
        __syncthreads();
        if (left > kGemvSeg) load_x(c0 + kGemvSeg, buf ^ 1u);
        const uint64_t next_word = row_word(c0 + kGemvSeg);
        const uint32_t pc = __popcll(word);
        const uint32_t incl = wave_inclusive_scan(pc);
        const uint32_t cnt = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(incl), 63));
        {
            uint32_t at = incl - pc;  // values of the segment before this lane's word
            uint32_t e8[8];
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const uint32_t byte = static_cast<uint32_t>(word >> (8 * b)) & 0xffu;
                e8[b] = (at << 8) | byte;
                at += __popc(byte);
            }
            u32x4 lo, hi;
            lo.x = e8[0];
            lo.y = e8[1];
            lo.z = e8[2];
            lo.w = e8[3];
            hi.x = e8[4];
            hi.y = e8[5];
            hi.z = e8[6];
            hi.w = e8[7];
            reinterpret_cast<u32x4 *>(entry)[2 * lane] = lo;
            reinterpret_cast<u32x4 *>(entry)[2 * lane + 1] = hi;
        }
        wave_lds_sync();
        const uintptr_t vseg = vbeg + 2 * next_value;
        if (windows_inside(vseg, vseg + 2 * uintptr_t(cnt), vbeg, vend)) {  // wave-uniform
            uint32_t e[kGemvSeg / 512];
            WindowLoad win[kGemvSeg / 512];
#pragma unroll
            for (int k = 0; k < kGemvSeg / 512; ++k) e[k] = entry[k * 64 + lane];
#pragma unroll
            for (int k = 0; k < kGemvSeg / 512; ++k) win[k] = window_issue(vseg + 2 * uintptr_t(e[k] >> 8));
#pragma unroll
            for (int k = 0; k < kGemvSeg / 512; ++k) {
                const u32x4 w = window_finish(win[k], vseg + 2 * uintptr_t(e[k] >> 8));
                sink(place_window(s_tables, e[k] & 0xffu, w), s_x[buf][k * 64 + lane]);
            }
        } else {  // a segment at the very beginning or end of `values`
#pragma unroll 1
            for (int k = 0; k < kGemvSeg / 512; ++k) {
                const uint32_t e = entry[k * 64 + lane];
                const u32x4 w = window_guarded(vseg + 2 * uintptr_t(e >> 8), vbeg, vend);
                sink(place_window(s_tables, e & 0xffu, w), s_x[buf][k * 64 + lane]);
            }
        }
        wave_lds_sync();  // the next segment's entries stay behind this segment's reads
        next_value += cnt;
        word = next_word;
    }
    const float total = wave_sum_f32(sink.acc);
    if (lane == 0 && row_ok) G.y[i] = total;
}

// ---------------------------------------------------------------- device-side compression

// 16 bytes of the dense matrix: elements [le, le + kLaneElems) of a tile that has
// `nvalid` elements; elements past the end read as zero.
template <int E, bool kAlignedIn>
__device__ __forceinline__ u32x4 load_dense16(const uint8_t *tile_in, uint32_t le, uint32_t nvalid) {
    if (kAlignedIn && le + Shape<E>::kLaneElems <= nvalid)
        return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(tile_in + size_t(le) * E));
    uint32_t d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < Shape<E>::kLaneElems; ++j) {
        uint32_t v = 0;
        if (le + j < nvalid)
            v = (E == 2) ? uint32_t(reinterpret_cast<const uint16_t *>(tile_in)[le + j]) : uint32_t(tile_in[le + j]);
        d[(E * j) >> 2] |= v << (8 * ((E * j) & 3));
    }
    u32x4 r;
    r.x = d[0];
    r.y = d[1];
    r.z = d[2];
    r.w = d[3];
    return r;
}

// A lane's kSteps 16-byte pieces of a tile of the dense matrix.  A whole, aligned tile is one
// wave-uniform case with unconditional loads, all issued before the first is used (under a
// per-piece bounds test the compiler waits after every load); only the ragged last tile and
// unaligned inputs go piece by piece.
template <int E, bool kAlignedIn>
__device__ __forceinline__ void load_dense_tile(const uint8_t *tile_in, uint32_t lane, uint32_t nvalid,
                                                u32x4 (&d)[Shape<E>::kSteps]) {
    using Sh = Shape<E>;
    if (kAlignedIn && nvalid == kTileElems) {
#pragma unroll
        for (int k = 0; k < Sh::kSteps; ++k)
            d[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(tile_in) + k * 64 + lane);
    } else {
#pragma unroll
        for (int k = 0; k < Sh::kSteps; ++k) d[k] = load_dense16<E, kAlignedIn>(tile_in, (k * 64 + lane) * Sh::kLaneElems, nvalid);
    }
}

// bit j = (element j of the 16 bytes is not the all-zero pattern)
template <int E>
__device__ __forceinline__ uint32_t nonzero_bits(u32x4 d) {
    const uint32_t dd[4] = {d.x, d.y, d.z, d.w};
    uint32_t bits = 0;
#pragma unroll
    for (int j = 0; j < Shape<E>::kLaneElems; ++j) {
        const uint32_t v = (dd[(E * j) >> 2] >> (8 * ((E * j) & 3))) & ((E == 2) ? 0xffffu : 0xffu);
        bits |= (v != 0 ? 1u : 0u) << j;
    }
    return bits;
}

struct CompressParams {
    const void *dense;
    uint64_t *bitmap;
    void *values;
    int64_t n;
    int64_t capacity;  // elements `values` has room for
    MatParams table;   // chunk_total / tile_off of this matrix (bitmap, n filled in as well)
};

// Algorithm 1, step 1 on the device: the position bitmap.  One wave per tile; the lane
// bit groups of the 4096 elements are assembled into 64-bit words through LDS.
template <int E, bool kAlignedIn>
__global__ __launch_bounds__(64) void endor_mask_kernel(CompressParams C) {
    using Sh = Shape<E>;
    __shared__ uint64_t s_words[kTileWords];
    const uint32_t lane = threadIdx.x;
    const int64_t tile = blockIdx.x;
    const int64_t e0 = tile * kTileElems;
    const int64_t left = C.n - e0;
    const uint32_t nvalid = left < kTileElems ? static_cast<uint32_t>(left) : uint32_t(kTileElems);
    const uint8_t *tile_in = reinterpret_cast<const uint8_t *>(C.dense) + e0 * E;
    u32x4 d[Sh::kSteps];
    load_dense_tile<E, kAlignedIn>(tile_in, lane, nvalid, d);
#pragma unroll
    for (int k = 0; k < Sh::kSteps; ++k) {
        const uint32_t bits = nonzero_bits<E>(d[k]);
        if (E == 2)
            reinterpret_cast<uint8_t *>(s_words)[k * 64 + lane] = static_cast<uint8_t>(bits);
        else
            reinterpret_cast<uint16_t *>(s_words)[k * 64 + lane] = static_cast<uint16_t>(bits);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int64_t w = tile * kTileWords + lane;
    if (w < ((C.n + 63) >> 6)) C.bitmap[w] = s_words[lane];  // pad bits are zero: elements past n read as zero
}

// Algorithm 1, step 2 on the device: pack the non-zero elements of one tile at the
// tile's offset.  The values are scattered into LDS at rank order and written out in
// 16-byte units; the units a tile shares with its neighbours (first and last) are
// written element by element so that each element of `values` has exactly one writer.
template <int E, bool kAlignedIn>
__global__ __launch_bounds__(64) void endor_pack_kernel(CompressParams C) {
    using Sh = Shape<E>;
    __shared__ WaveScratch<E> S;
    const uint32_t lane = threadIdx.x;
    const int64_t tile = blockIdx.x;
    // the tile's elements first: their loads are in flight while the table is looked up
    const int64_t e0 = tile * kTileElems;
    const int64_t left = C.n - e0;
    const uint32_t nvalid = left < kTileElems ? static_cast<uint32_t>(left) : uint32_t(kTileElems);
    const uint8_t *tile_in = reinterpret_cast<const uint8_t *>(C.dense) + e0 * E;
    u32x4 d[Sh::kSteps];
    load_dense_tile<E, kAlignedIn>(tile_in, lane, nvalid, d);

    const MatParams &M = C.table;
    const uint32_t c = static_cast<uint32_t>(tile / kTilesPerChunk);
    const uint32_t tl = static_cast<uint32_t>(tile % kTilesPerChunk);
    const uint32_t *tile_off = M.tile_off + size_t(c) * kChunkStride + tl;
    const uint32_t o0 = tile_off[0];
    uint32_t cnt = tile_off[1] - o0;
    cnt = cnt > kTileElems ? kTileElems : cnt;
    const uint64_t first = chunk_base(M.chunk_total, c, lane) + o0;  // index of the tile's first value

    const uintptr_t vbase = reinterpret_cast<uintptr_t>(C.values);
    const uintptr_t vaddr = vbase + E * first;
    const uintptr_t a16 = vaddr & ~uintptr_t(15);
    const uint32_t shift = static_cast<uint32_t>(vaddr - a16) / E;

    // word popcounts from the data itself (the same bits endor_mask_kernel wrote)
    uint32_t bits[Sh::kSteps];
#pragma unroll
    for (int k = 0; k < Sh::kSteps; ++k) {
        bits[k] = nonzero_bits<E>(d[k]);
        if (E == 2)
            reinterpret_cast<uint8_t *>(S.words)[k * 64 + lane] = static_cast<uint8_t>(bits[k]);
        else
            reinterpret_cast<uint16_t *>(S.words)[k * 64 + lane] = static_cast<uint16_t>(bits[k]);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint64_t word = S.words[lane];
    const uint32_t pc = __popcll(word);
    const uint32_t incl = wave_inclusive_scan(pc);
    S.start[lane] = incl - pc + shift;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // scatter the non-zero elements into LDS in rank order
#pragma unroll
    for (int k = 0; k < Sh::kSteps; ++k) {
        const uint32_t wi = k * Sh::kLaneElems + lane / Sh::kLanesPerWord;
        const uint64_t w = S.words[wi];
        const uint32_t sh = (lane % Sh::kLanesPerWord) * Sh::kLaneElems;
        const uint32_t s = S.start[wi] + __popcll(w & ((uint64_t(1) << sh) - 1));
        const uint32_t dd[4] = {d[k].x, d[k].y, d[k].z, d[k].w};
#pragma unroll
        for (int j = 0; j < Sh::kLaneElems; ++j) {
            if ((bits[k] >> j) & 1u) {
                const uint32_t idx = s + __popc(bits[k] & ((1u << j) - 1));
                const uint32_t v = dd[(E * j) >> 2] >> (8 * ((E * j) & 3));
                if (E == 2)
                    reinterpret_cast<uint16_t *>(S.stage)[idx] = static_cast<uint16_t>(v);
                else
                    reinterpret_cast<uint8_t *>(S.stage)[idx] = static_cast<uint8_t>(v);
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // write the slice out: elements [shift, shift + cnt) of the staging area go to
    // values[first, first + cnt), never past `capacity`
    const uint32_t nch = cnt ? (((shift + cnt) * E + 15) >> 4) : 0;
    const int64_t room = C.capacity - static_cast<int64_t>(first);  // elements this tile may write
    for (uint32_t ch = lane; ch < nch; ch += 64) {
        const uint32_t el0 = ch * Sh::kLaneElems;  // staging index of the unit's first element
        const bool inside = el0 >= shift && el0 + Sh::kLaneElems <= shift + cnt &&
                            static_cast<int64_t>(el0 + Sh::kLaneElems - shift) <= room;
        if (inside) {
            *global_ptr_mut<u32x4>(a16 + 16 * uintptr_t(ch)) = S.stage[ch];
        } else {
#pragma unroll
            for (int j = 0; j < Sh::kLaneElems; ++j) {
                const uint32_t el = el0 + j;
                if (el >= shift && el < shift + cnt && static_cast<int64_t>(el - shift) < room) {
                    if (E == 2)
                        global_ptr_mut<uint16_t>(a16)[el] = reinterpret_cast<const uint16_t *>(S.stage)[el];
                    else
                        global_ptr_mut<uint8_t>(a16)[el] = reinterpret_cast<const uint8_t *>(S.stage)[el];
                }
            }
        }
    }
}

// total number of 1 bits of a matrix whose table has been built: one wave
__global__ __launch_bounds__(64) void endor_total_kernel(MatParams M, int64_t *__restrict__ nnz_out) {
    const uint64_t total = chunk_base(M.chunk_total, M.nchunks, threadIdx.x);
    if (threadIdx.x == 0) *nnz_out = static_cast<int64_t>(total);
}

// Check mode: one wave per matrix compares nnz with the number of 1 bits the table records.
__global__ __launch_bounds__(64) void endor_check_kernel(BatchParams P, int32_t *__restrict__ status) {
    const MatParams &M = P.m[blockIdx.x];
    const uint64_t total = chunk_base(M.chunk_total, M.nchunks, threadIdx.x);
    if (threadIdx.x == 0)
        status[M.chunk_begin] = total == static_cast<uint64_t>(M.nnz) ? ENDOR_OK : ENDOR_ERR_NNZ_MISMATCH;
}

// ---------------------------------------------------------------- kernel 3: row offsets

// One wave per row start: rank(i*cols) = chunk start + tile offset + 1 bits of the
// tile's words below the position.  Entry `rows` is the total number of 1 bits.
__global__ __launch_bounds__(kBlock) void endor_row_offsets_kernel(MatParams M, int64_t rows, int64_t cols,
                                                                   int64_t *__restrict__ row_offsets) {
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    const int64_t i = int64_t(blockIdx.x) * kWaves + wave;
    if (i > rows) return;
    const int64_t e = i * cols;  // == n for i == rows
    const int64_t ntiles = (M.n + kTileElems - 1) / kTileElems;
    int64_t tile = e >> 12;
    uint64_t rank;
    if (tile >= ntiles) {
        // position n when n is a multiple of the tile size: everything counts
        rank = chunk_base(M.chunk_total, M.nchunks, lane);
    } else {
        const uint32_t c = static_cast<uint32_t>(tile / kTilesPerChunk);
        const uint32_t tl = static_cast<uint32_t>(tile % kTilesPerChunk);
        rank = chunk_base(M.chunk_total, c, lane) + M.tile_off[size_t(c) * kChunkStride + tl];
        const int64_t w = tile * kTileWords + lane;
        const int64_t we = e >> 6;  // word holding position e
        uint64_t word = 0;
        if (w <= we) word = load_word_guarded(M.bitmap, w, M.n >> 6, static_cast<uint32_t>(M.n & 63));
        if (w == we) word &= (uint64_t(1) << (e & 63)) - 1;
        rank += wave_sum(__popcll(word));
    }
    if (lane == 0) row_offsets[i] = static_cast<int64_t>(rank);
}

// ---------------------------------------------------------------- host side

struct Group {
    BatchParams P;
    uint32_t chunks = 0;
    bool aligned_out = true;
    int64_t elems = 0, nnz = 0;  // totals over the group (launch heuristics only)
};

enum Need { kNeedBitmap = 1, kNeedValuesDense = 2 };

// Validate `count` matrices starting at the workspace offset *ws_off and fill one
// launch group.  Advances *ws_off past the slices it used.
endor_status fill_group(const endor_matrix *mats, int count, int need, int elem_bytes, char *ws,
                        size_t ws_bytes, size_t *ws_off, Group *g) {
    const uintptr_t elem_mask = static_cast<uintptr_t>(elem_bytes - 1);
    g->P.count = 0;
    for (int i = 0; i < ENDOR_MAX_BATCH; ++i) g->P.first_chunk[i] = 0xffffffffu;
    g->chunks = 0;
    g->aligned_out = true;
    g->elems = 0;
    g->nnz = 0;
    for (int i = 0; i < count; ++i) {
        const endor_matrix &m = mats[i];
        if (m.rows < 0 || m.cols < 0) return ENDOR_ERR_INVALID_ARG;
        if (!dims_ok(m.rows, m.cols)) return ENDOR_ERR_UNSUPPORTED;
        const int64_t n = m.rows * m.cols;
        if (n == 0) continue;
        if (!m.d_bitmap || (reinterpret_cast<uintptr_t>(m.d_bitmap) & 7)) return ENDOR_ERR_INVALID_ARG;
        if (need & kNeedValuesDense) {
            if (m.nnz < 0 || m.nnz > n) return ENDOR_ERR_INVALID_ARG;
            if (!m.d_dense || (reinterpret_cast<uintptr_t>(m.d_dense) & elem_mask)) return ENDOR_ERR_INVALID_ARG;
            if (m.nnz > 0 && (!m.d_values || (reinterpret_cast<uintptr_t>(m.d_values) & elem_mask)))
                return ENDOR_ERR_INVALID_ARG;
            if (reinterpret_cast<uintptr_t>(m.d_dense) & 15) g->aligned_out = false;
        }
        const uint32_t nc = chunks_of(n);
        const size_t need_bytes = workspace_bytes_n(n);
        if (*ws_off + need_bytes > ws_bytes) return ENDOR_ERR_BUFFER_TOO_SMALL;
        MatParams &M = g->P.m[g->P.count++];
        M.bitmap = reinterpret_cast<const uint64_t *>(m.d_bitmap);
        M.values = m.d_values;
        M.dense = m.d_dense;
        M.chunk_total = reinterpret_cast<uint32_t *>(ws + *ws_off);
        M.tile_off = reinterpret_cast<uint32_t *>(ws + *ws_off + align256(nc * sizeof(uint32_t)));
        M.n = n;
        M.nnz = m.nnz;
        M.chunk_begin = g->chunks;
        g->P.first_chunk[g->P.count - 1] = g->chunks;
        M.nchunks = nc;
        g->chunks += nc;
        g->elems += n;
        g->nnz += m.nnz;
        *ws_off += need_bytes;
    }
    return ENDOR_OK;
}

template <int E>
void launch_expand(const Group &g, hipStream_t s) {
    const dim3 grid(g.chunks * kTilesPerChunk);
    if (!g.aligned_out)
        hipLaunchKernelGGL((endor_expand_kernel<E, false, kTileElems, false>), grid, dim3(64), 0, s, g.P);
    else if (g.nnz * 5 < g.elems)  // fewer than one element in five kept: store-dominated
        hipLaunchKernelGGL((endor_expand_kernel<E, true, 1024, true>), grid, dim3(64), 0, s, g.P);
    else
        hipLaunchKernelGGL((endor_expand_kernel<E, true, kTileElems, false>), grid, dim3(64), 0, s, g.P);
}

// The shared driver of every device entry point.  `mats` holds 16-bit typed pointers;
// with elem_bytes == 1 they are really 8-bit (endor_matrix_u8 has the same layout).
endor_status run_batch(const endor_matrix *mats, int count, void *d_workspace, size_t workspace_bytes,
                       void *stream, bool build, bool expand, int elem_bytes = 2) {
    if (count < 0 || (count > 0 && !mats)) return ENDOR_ERR_INVALID_ARG;
    if (count == 0) return ENDOR_OK;
    for (int i = 0; i < count; ++i) {
        if (mats[i].rows < 0 || mats[i].cols < 0) return ENDOR_ERR_INVALID_ARG;
        if (!dims_ok(mats[i].rows, mats[i].cols)) return ENDOR_ERR_UNSUPPORTED;
    }
    // a batch of empty matrices needs no workspace; anything else needs an aligned one
    if (endor_batch_workspace_bytes(mats, count) != 0 &&
        (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 255)))
        return ENDOR_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(d_workspace);
    const int need = kNeedBitmap | (expand ? kNeedValuesDense : 0);

    // validate everything before the first launch
    {
        size_t off = 0;
        Group g;
        for (int b = 0; b < count; b += ENDOR_MAX_BATCH) {
            const int nb = count - b < ENDOR_MAX_BATCH ? count - b : ENDOR_MAX_BATCH;
            endor_status st = fill_group(mats + b, nb, need, elem_bytes, ws, workspace_bytes, &off, &g);
            if (st != ENDOR_OK) return st;
        }
    }
    size_t off = 0;
    Group g;
    for (int b = 0; b < count; b += ENDOR_MAX_BATCH) {
        const int nb = count - b < ENDOR_MAX_BATCH ? count - b : ENDOR_MAX_BATCH;
        fill_group(mats + b, nb, need, elem_bytes, ws, workspace_bytes, &off, &g);
        if (g.chunks == 0) continue;
        if (build) {
            hipLaunchKernelGGL(endor_tile_offsets_kernel, dim3(g.chunks), dim3(kCountBlock), 0, s, g.P);
            if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
        }
        if (expand) {
            if (elem_bytes == 2)
                launch_expand<2>(g, s);
            else
                launch_expand<1>(g, s);
            if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
        }
    }
    return ENDOR_OK;
}

endor_matrix one_matrix(int64_t rows, int64_t cols, const uint8_t *d_bitmap, const uint16_t *d_values,
                        int64_t nnz, uint16_t *d_dense) {
    endor_matrix m;
    m.rows = rows;
    m.cols = cols;
    m.d_bitmap = d_bitmap;
    m.d_values = d_values;
    m.nnz = nnz;
    m.d_dense = d_dense;
    return m;
}

}  // namespace

extern "C" size_t endor_workspace_bytes(int64_t rows, int64_t cols) {
    if (!dims_ok(rows, cols)) return 0;
    return workspace_bytes_n(rows * cols);
}

extern "C" size_t endor_batch_workspace_bytes(const endor_matrix *mats, int count) {
    if (count < 0 || (count > 0 && !mats)) return 0;
    size_t total = 0;
    for (int i = 0; i < count; ++i) {
        if (!dims_ok(mats[i].rows, mats[i].cols)) return 0;
        total += workspace_bytes_n(mats[i].rows * mats[i].cols);
    }
    return total;
}

extern "C" endor_status endor_build_offsets_batch(const endor_matrix *mats, int count, void *d_workspace,
                                                  size_t workspace_bytes, void *stream) {
    return run_batch(mats, count, d_workspace, workspace_bytes, stream, true, false);
}

extern "C" endor_status endor_decompress_batch(const endor_matrix *mats, int count, void *d_workspace,
                                               size_t workspace_bytes, void *stream) {
    return run_batch(mats, count, d_workspace, workspace_bytes, stream, true, true);
}

extern "C" endor_status endor_decompress_batch_with_offsets(const endor_matrix *mats, int count,
                                                            const void *d_workspace, size_t workspace_bytes,
                                                            void *stream) {
    return run_batch(mats, count, const_cast<void *>(d_workspace), workspace_bytes, stream, false, true);
}

extern "C" endor_status endor_check_batch(const endor_matrix *mats, int count, const void *d_workspace,
                                          size_t workspace_bytes, int32_t *d_status, void *stream) {
    if (count < 0 || (count > 0 && (!mats || !d_status))) return ENDOR_ERR_INVALID_ARG;
    if (count == 0) return ENDOR_OK;
    if (reinterpret_cast<uintptr_t>(d_status) & 3) return ENDOR_ERR_INVALID_ARG;
    for (int i = 0; i < count; ++i) {
        if (mats[i].rows < 0 || mats[i].cols < 0 || mats[i].nnz < 0) return ENDOR_ERR_INVALID_ARG;
        if (!dims_ok(mats[i].rows, mats[i].cols)) return ENDOR_ERR_UNSUPPORTED;
    }
    if (endor_batch_workspace_bytes(mats, count) != 0 &&
        (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 255)))
        return ENDOR_ERR_INVALID_ARG;
    if (endor_batch_workspace_bytes(mats, count) > workspace_bytes) return ENDOR_ERR_BUFFER_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = const_cast<char *>(static_cast<const char *>(d_workspace));
    size_t off = 0;
    for (int b = 0; b < count; b += ENDOR_MAX_BATCH) {
        const int nb = count - b < ENDOR_MAX_BATCH ? count - b : ENDOR_MAX_BATCH;
        // one descriptor per matrix, empty ones included (they have no chunks and no 1 bits);
        // chunk_begin carries the matrix's index inside the batch for the kernel
        BatchParams P;
        P.count = nb;
        for (int i = 0; i < ENDOR_MAX_BATCH; ++i) P.first_chunk[i] = 0xffffffffu;  // not used by the check kernel
        for (int i = 0; i < nb; ++i) {
            const endor_matrix &m = mats[b + i];
            const int64_t n = m.rows * m.cols;
            MatParams &M = P.m[i];
            M = MatParams{};
            M.n = n;
            M.nnz = m.nnz;
            M.nchunks = n > 0 ? chunks_of(n) : 0;
            M.chunk_total = reinterpret_cast<uint32_t *>(ws + off);
            M.chunk_begin = static_cast<uint32_t>(b + i);
            off += n > 0 ? workspace_bytes_n(n) : 0;
        }
        hipLaunchKernelGGL(endor_check_kernel, dim3(nb), dim3(64), 0, s, P, d_status);
        if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
    }
    return ENDOR_OK;
}

extern "C" endor_status endor_decompress(int64_t rows, int64_t cols, const uint8_t *d_bitmap,
                                         const uint16_t *d_values, int64_t nnz, void *d_workspace,
                                         size_t workspace_bytes, uint16_t *d_dense, void *stream) {
    const endor_matrix m = one_matrix(rows, cols, d_bitmap, d_values, nnz, d_dense);
    return run_batch(&m, 1, d_workspace, workspace_bytes, stream, true, true);
}

extern "C" endor_status endor_decompress_with_offsets(int64_t rows, int64_t cols, const uint8_t *d_bitmap,
                                                      const uint16_t *d_values, int64_t nnz,
                                                      const void *d_workspace, size_t workspace_bytes,
                                                      uint16_t *d_dense, void *stream) {
    const endor_matrix m = one_matrix(rows, cols, d_bitmap, d_values, nnz, d_dense);
    return run_batch(&m, 1, const_cast<void *>(d_workspace), workspace_bytes, stream, false, true);
}

extern "C" endor_status endor_build_offsets(int64_t rows, int64_t cols, const uint8_t *d_bitmap,
                                            void *d_workspace, size_t workspace_bytes,
                                            int64_t *d_row_offsets, void *stream) {
    const endor_matrix m = one_matrix(rows, cols, d_bitmap, nullptr, 0, nullptr);
    if (d_row_offsets && (reinterpret_cast<uintptr_t>(d_row_offsets) & 7)) return ENDOR_ERR_INVALID_ARG;
    endor_status st = run_batch(&m, 1, d_workspace, workspace_bytes, stream, true, false);
    if (st != ENDOR_OK || !d_row_offsets) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t n = rows * cols;
    MatParams M{};
    if (n > 0) {
        size_t off = 0;
        Group g;
        fill_group(&m, 1, kNeedBitmap, 2, static_cast<char *>(d_workspace), workspace_bytes, &off, &g);
        M = g.P.m[0];
    }
    // n == 0: nchunks == 0 and every position is >= ntiles, so all entries are 0
    const int64_t entries = rows + 1;
    if ((entries + kWaves - 1) / kWaves > 0x7fffffff) return ENDOR_ERR_UNSUPPORTED;
    const unsigned blocks = static_cast<unsigned>((entries + kWaves - 1) / kWaves);
    hipLaunchKernelGGL(endor_row_offsets_kernel, dim3(blocks), dim3(kBlock), 0, s, M, rows, cols, d_row_offsets);
    if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
    return ENDOR_OK;
}

// ---------------------------------------------------------------- no-allocation variant

namespace {

// The offset tables of endor_decompress_batch_static live here instead of in a caller's
// workspace.  Every device the library runs on holds its own copy of the array at its own
// address; in host code the array's name is only a handle for hipGetSymbolAddress, never
// a device address.
static __device__ __align__(256) unsigned char scratch[ENDOR_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once known

// Device address of `scratch` on the current device, resolved on the first call per device.
endor_status static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return ENDOR_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return ENDOR_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ENDOR_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ENDOR_OK;
}

}  // namespace

extern "C" endor_status endor_decompress_batch_static(const endor_matrix *mats, int count, void *stream) {
    if (count < 0 || (count > 0 && !mats)) return ENDOR_ERR_INVALID_ARG;
    if (count == 0) return ENDOR_OK;
    for (int i = 0; i < count; ++i) {
        if (mats[i].rows < 0 || mats[i].cols < 0) return ENDOR_ERR_INVALID_ARG;
        if (!dims_ok(mats[i].rows, mats[i].cols)) return ENDOR_ERR_UNSUPPORTED;
    }
    const size_t need = endor_batch_workspace_bytes(mats, count);
    if (need > size_t(ENDOR_STATIC_SCRATCH_BYTES)) return ENDOR_ERR_BUFFER_TOO_SMALL;
    void *ws = nullptr;
    const endor_status st = static_scratch(&ws);
    if (st != ENDOR_OK) return st;
    // Nothing in the table has to start at zero: the tile-offset kernel writes every entry
    // of every chunk of this batch before the expand kernel reads it.
    return run_batch(mats, count, ws, size_t(ENDOR_STATIC_SCRATCH_BYTES), stream, true, true);
}

// ---------------------------------------------------------------- 8-bit elements (Section 4.2)

static_assert(sizeof(endor_matrix_u8) == sizeof(endor_matrix), "same descriptor layout for both widths");

extern "C" endor_status endor_decompress_u8(int64_t rows, int64_t cols, const uint8_t *d_bitmap,
                                            const uint8_t *d_values, int64_t nnz, void *d_workspace,
                                            size_t workspace_bytes, uint8_t *d_dense, void *stream) {
    const endor_matrix m = one_matrix(rows, cols, d_bitmap, reinterpret_cast<const uint16_t *>(d_values), nnz,
                                      reinterpret_cast<uint16_t *>(d_dense));
    return run_batch(&m, 1, d_workspace, workspace_bytes, stream, true, true, 1);
}

extern "C" endor_status endor_decompress_u8_with_offsets(int64_t rows, int64_t cols, const uint8_t *d_bitmap,
                                                         const uint8_t *d_values, int64_t nnz,
                                                         const void *d_workspace, size_t workspace_bytes,
                                                         uint8_t *d_dense, void *stream) {
    const endor_matrix m = one_matrix(rows, cols, d_bitmap, reinterpret_cast<const uint16_t *>(d_values), nnz,
                                      reinterpret_cast<uint16_t *>(d_dense));
    return run_batch(&m, 1, const_cast<void *>(d_workspace), workspace_bytes, stream, false, true, 1);
}

extern "C" endor_status endor_decompress_batch_u8(const endor_matrix_u8 *mats, int count, void *d_workspace,
                                                  size_t workspace_bytes, void *stream) {
    return run_batch(reinterpret_cast<const endor_matrix *>(mats), count, d_workspace, workspace_bytes, stream,
                     true, true, 1);
}

extern "C" endor_status endor_decompress_batch_u8_with_offsets(const endor_matrix_u8 *mats, int count,
                                                               const void *d_workspace, size_t workspace_bytes,
                                                               void *stream) {
    return run_batch(reinterpret_cast<const endor_matrix *>(mats), count, const_cast<void *>(d_workspace),
                     workspace_bytes, stream, false, true, 1);
}

// ---------------------------------------------------------------- selected rows (Section 4.2)

namespace {

endor_status run_rows(int elem_bytes, int64_t rows, int64_t cols, const uint8_t *d_bitmap, const void *d_values,
                      int64_t nnz, const int64_t *d_row_offsets, const int64_t *d_sel, int64_t nsel, void *d_out,
                      void *stream) {
    if (rows < 0 || cols < 0 || nsel < 0 || nnz < 0) return ENDOR_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols)) return ENDOR_ERR_UNSUPPORTED;
    if (nsel == 0 || cols == 0) return ENDOR_OK;
    if (nsel > kMaxElems / cols) return ENDOR_ERR_UNSUPPORTED;
    const uintptr_t em = static_cast<uintptr_t>(elem_bytes - 1);
    if (nnz > rows * cols) return ENDOR_ERR_INVALID_ARG;
    if (!d_bitmap || (reinterpret_cast<uintptr_t>(d_bitmap) & 7)) return ENDOR_ERR_INVALID_ARG;
    if (nnz > 0 && (!d_values || (reinterpret_cast<uintptr_t>(d_values) & em))) return ENDOR_ERR_INVALID_ARG;
    if (!d_row_offsets || (reinterpret_cast<uintptr_t>(d_row_offsets) & 7)) return ENDOR_ERR_INVALID_ARG;
    if (!d_sel || (reinterpret_cast<uintptr_t>(d_sel) & 7)) return ENDOR_ERR_INVALID_ARG;
    if (!d_out || (reinterpret_cast<uintptr_t>(d_out) & em)) return ENDOR_ERR_INVALID_ARG;
    RowsParams R;
    R.bitmap = reinterpret_cast<const uint64_t *>(d_bitmap);
    R.values = d_values;
    R.out = d_out;
    R.row_offsets = d_row_offsets;
    R.sel = d_sel;
    R.rows = rows;
    R.cols = cols;
    R.nnz = nnz;
    R.nsel = nsel;
    R.segs = static_cast<uint32_t>((cols + kTileElems - 1) / kTileElems);
    const int64_t blocks = nsel * R.segs;
    if (blocks > 0x7fffffff) return ENDOR_ERR_UNSUPPORTED;
    // every segment start (r*cols + g*4096 elements) is 16-byte aligned iff the row pitch is
    const bool aligned = (reinterpret_cast<uintptr_t>(d_out) & 15) == 0 && (cols * elem_bytes) % 16 == 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid(static_cast<unsigned>(blocks));
    // A selection is usually small (Section 4.2: the rows of the active neurons), so the kernel
    // lives on how many waves a compute unit holds at once: when no more than 9 elements in 16 are
    // kept overall, a staging area of 2304 values (a tile with more takes the step-by-step path)
    // lets 29 waves share a unit instead of 17.
    const bool small_stage = nnz <= (rows * cols / 16) * 9;
    if (elem_bytes == 2) {
        if (aligned && small_stage)
            hipLaunchKernelGGL((endor_expand_rows_kernel<2, true, 2304>), grid, dim3(64), 0, s, R);
        else if (aligned)
            hipLaunchKernelGGL((endor_expand_rows_kernel<2, true>), grid, dim3(64), 0, s, R);
        else
            hipLaunchKernelGGL((endor_expand_rows_kernel<2, false>), grid, dim3(64), 0, s, R);
    } else {
        if (aligned)
            hipLaunchKernelGGL((endor_expand_rows_kernel<1, true>), grid, dim3(64), 0, s, R);
        else
            hipLaunchKernelGGL((endor_expand_rows_kernel<1, false>), grid, dim3(64), 0, s, R);
    }
    if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
    return ENDOR_OK;
}

}  // namespace

extern "C" endor_status endor_decompress_rows(int64_t rows, int64_t cols, const uint8_t *d_bitmap,
                                              const uint16_t *d_values, int64_t nnz,
                                              const int64_t *d_row_offsets, const int64_t *d_sel, int64_t nsel,
                                              uint16_t *d_out, void *stream) {
    return run_rows(2, rows, cols, d_bitmap, d_values, nnz, d_row_offsets, d_sel, nsel, d_out, stream);
}

extern "C" endor_status endor_decompress_rows_u8(int64_t rows, int64_t cols, const uint8_t *d_bitmap,
                                                 const uint8_t *d_values, int64_t nnz,
                                                 const int64_t *d_row_offsets, const int64_t *d_sel,
                                                 int64_t nsel, uint8_t *d_out, void *stream) {
    return run_rows(1, rows, cols, d_bitmap, d_values, nnz, d_row_offsets, d_sel, nsel, d_out, stream);
}

// ---------------------------------------------------------------- device-side compression

namespace {

template <int E>
endor_status run_compress_device(int64_t rows, int64_t cols, const void *d_dense, uint8_t *d_bitmap,
                                 void *d_values, int64_t values_capacity, void *d_workspace,
                                 size_t workspace_bytes, int64_t *d_row_offsets, int64_t *d_nnz_out,
                                 void *stream) {
    if (rows < 0 || cols < 0 || values_capacity < 0) return ENDOR_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols)) return ENDOR_ERR_UNSUPPORTED;
    if (!d_nnz_out || (reinterpret_cast<uintptr_t>(d_nnz_out) & 7)) return ENDOR_ERR_INVALID_ARG;
    if (d_row_offsets && (reinterpret_cast<uintptr_t>(d_row_offsets) & 7)) return ENDOR_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t n = rows * cols;
    const uintptr_t em = E - 1;
    if (n > 0) {
        if (!d_dense || (reinterpret_cast<uintptr_t>(d_dense) & em)) return ENDOR_ERR_INVALID_ARG;
        if (!d_bitmap || (reinterpret_cast<uintptr_t>(d_bitmap) & 7)) return ENDOR_ERR_INVALID_ARG;
        if (values_capacity > 0 && (!d_values || (reinterpret_cast<uintptr_t>(d_values) & em)))
            return ENDOR_ERR_INVALID_ARG;
        if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 255)) return ENDOR_ERR_INVALID_ARG;
        if (workspace_bytes < workspace_bytes_n(n)) return ENDOR_ERR_BUFFER_TOO_SMALL;
    }
    // the table (and the row offsets) come from the ordinary offsets path, run on the
    // bitmap the mask kernel writes
    CompressParams C{};
    C.dense = d_dense;
    C.bitmap = reinterpret_cast<uint64_t *>(d_bitmap);
    C.values = d_values;
    C.n = n;
    C.capacity = values_capacity;
    const bool aligned_in = (reinterpret_cast<uintptr_t>(d_dense) & 15) == 0;
    const unsigned ntiles = static_cast<unsigned>((n + kTileElems - 1) / kTileElems);
    if (n > 0) {
        if (aligned_in)
            hipLaunchKernelGGL((endor_mask_kernel<E, true>), dim3(ntiles), dim3(64), 0, s, C);
        else
            hipLaunchKernelGGL((endor_mask_kernel<E, false>), dim3(ntiles), dim3(64), 0, s, C);
        if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
    }
    endor_status st = endor_build_offsets(rows, cols, d_bitmap, d_workspace, workspace_bytes, d_row_offsets, stream);
    if (st != ENDOR_OK) return st;
    if (n > 0) {
        const endor_matrix m = one_matrix(rows, cols, d_bitmap, nullptr, 0, nullptr);
        size_t off = 0;
        Group g;
        fill_group(&m, 1, kNeedBitmap, E, static_cast<char *>(d_workspace), workspace_bytes, &off, &g);
        C.table = g.P.m[0];
        if (aligned_in)
            hipLaunchKernelGGL((endor_pack_kernel<E, true>), dim3(ntiles), dim3(64), 0, s, C);
        else
            hipLaunchKernelGGL((endor_pack_kernel<E, false>), dim3(ntiles), dim3(64), 0, s, C);
        if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
    }
    hipLaunchKernelGGL(endor_total_kernel, dim3(1), dim3(64), 0, s, C.table, d_nnz_out);
    if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
    return ENDOR_OK;
}

}  // namespace

extern "C" endor_status endor_compress_device(int64_t rows, int64_t cols, const uint16_t *d_dense,
                                              uint8_t *d_bitmap, uint16_t *d_values, int64_t values_capacity,
                                              void *d_workspace, size_t workspace_bytes,
                                              int64_t *d_row_offsets, int64_t *d_nnz_out, void *stream) {
    return run_compress_device<2>(rows, cols, d_dense, d_bitmap, d_values, values_capacity, d_workspace,
                                  workspace_bytes, d_row_offsets, d_nnz_out, stream);
}

extern "C" endor_status endor_compress_device_u8(int64_t rows, int64_t cols, const uint8_t *d_dense,
                                                 uint8_t *d_bitmap, uint8_t *d_values, int64_t values_capacity,
                                                 void *d_workspace, size_t workspace_bytes,
                                                 int64_t *d_row_offsets, int64_t *d_nnz_out, void *stream) {
    return run_compress_device<1>(rows, cols, d_dense, d_bitmap, d_values, values_capacity, d_workspace,
                                  workspace_bytes, d_row_offsets, d_nnz_out, stream);
}

// ---------------------------------------------------------------- fused consumer

extern "C" endor_status endor_gemv_f16(int64_t rows, int64_t cols, const uint8_t *d_bitmap,
                                       const uint16_t *d_values, int64_t nnz, const int64_t *d_row_offsets,
                                       const uint16_t *d_x, float *d_y, void *stream) {
    if (rows < 0 || cols < 0 || nnz < 0) return ENDOR_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols)) return ENDOR_ERR_UNSUPPORTED;
    if (rows == 0) return ENDOR_OK;
    if (rows > 0x7fffffff) return ENDOR_ERR_UNSUPPORTED;
    if (!d_y || (reinterpret_cast<uintptr_t>(d_y) & 3)) return ENDOR_ERR_INVALID_ARG;
    if (!d_row_offsets || (reinterpret_cast<uintptr_t>(d_row_offsets) & 7)) return ENDOR_ERR_INVALID_ARG;
    if (cols > 0) {
        if (nnz > rows * cols) return ENDOR_ERR_INVALID_ARG;
        if (!d_bitmap || (reinterpret_cast<uintptr_t>(d_bitmap) & 7)) return ENDOR_ERR_INVALID_ARG;
        if (!d_x || (reinterpret_cast<uintptr_t>(d_x) & 1)) return ENDOR_ERR_INVALID_ARG;
        if (nnz > 0 && (!d_values || (reinterpret_cast<uintptr_t>(d_values) & 1))) return ENDOR_ERR_INVALID_ARG;
    }
    GemvParams G;
    G.bitmap = reinterpret_cast<const uint64_t *>(d_bitmap);
    G.values = d_values;
    G.row_offsets = d_row_offsets;
    G.x = d_x;
    G.y = d_y;
    G.rows = rows;
    G.cols = cols;
    G.nnz = nnz;
    const dim3 grid(static_cast<unsigned>((rows + kGemvWaves - 1) / kGemvWaves)), block(64 * kGemvWaves);
    if ((reinterpret_cast<uintptr_t>(d_x) & 15) == 0 && cols % 8 == 0)
        hipLaunchKernelGGL(endor_gemv_f16_kernel<true>, grid, block, 0, static_cast<hipStream_t>(stream), G);
    else
        hipLaunchKernelGGL(endor_gemv_f16_kernel<false>, grid, block, 0, static_cast<hipStream_t>(stream), G);
    if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
    return ENDOR_OK;
}

// ---------------------------------------------------------------- selected columns (Section 4.2)

namespace {

constexpr int64_t kMaxGatherCols = int64_t(1) << 18;  // the row's bitmap and its prefixes live in LDS (16 bytes per 64 columns)

endor_status run_cols(int elem_bytes, int64_t rows, int64_t cols, const uint8_t *d_bitmap, const void *d_values,
                      int64_t nnz, const int64_t *d_row_offsets, const int64_t *d_sel, int64_t nsel, void *d_out,
                      void *stream) {
    if (rows < 0 || cols < 0 || nsel < 0 || nnz < 0) return ENDOR_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols)) return ENDOR_ERR_UNSUPPORTED;
    if (nsel == 0 || rows == 0 || cols == 0) return ENDOR_OK;
    if (cols > kMaxGatherCols || rows > 0x7fffffff || nsel > kMaxElems / rows) return ENDOR_ERR_UNSUPPORTED;
    const uintptr_t em = static_cast<uintptr_t>(elem_bytes - 1);
    if (nnz > rows * cols) return ENDOR_ERR_INVALID_ARG;
    if (!d_bitmap || (reinterpret_cast<uintptr_t>(d_bitmap) & 7)) return ENDOR_ERR_INVALID_ARG;
    if (nnz > 0 && (!d_values || (reinterpret_cast<uintptr_t>(d_values) & em))) return ENDOR_ERR_INVALID_ARG;
    if (!d_row_offsets || (reinterpret_cast<uintptr_t>(d_row_offsets) & 7)) return ENDOR_ERR_INVALID_ARG;
    if (!d_sel || (reinterpret_cast<uintptr_t>(d_sel) & 7)) return ENDOR_ERR_INVALID_ARG;
    if (!d_out || (reinterpret_cast<uintptr_t>(d_out) & em)) return ENDOR_ERR_INVALID_ARG;
    ColsParams C;
    C.bitmap = reinterpret_cast<const uint64_t *>(d_bitmap);
    C.values = d_values;
    C.out = d_out;
    C.row_offsets = d_row_offsets;
    C.sel = d_sel;
    C.rows = rows;
    C.cols = cols;
    C.nnz = nnz;
    C.nsel = nsel;
    const size_t lds = static_cast<size_t>((cols + 63) / 64) * 4 * sizeof(uint32_t);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid(static_cast<unsigned>(rows));
    if (elem_bytes == 2)
        hipLaunchKernelGGL((endor_gather_cols_kernel<2>), grid, dim3(kBlock), lds, s, C);
    else
        hipLaunchKernelGGL((endor_gather_cols_kernel<1>), grid, dim3(kBlock), lds, s, C);
    if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
    return ENDOR_OK;
}

}  // namespace

extern "C" endor_status endor_decompress_cols(int64_t rows, int64_t cols, const uint8_t *d_bitmap,
                                              const uint16_t *d_values, int64_t nnz,
                                              const int64_t *d_row_offsets, const int64_t *d_sel, int64_t nsel,
                                              uint16_t *d_out, void *stream) {
    return run_cols(2, rows, cols, d_bitmap, d_values, nnz, d_row_offsets, d_sel, nsel, d_out, stream);
}

extern "C" endor_status endor_decompress_cols_u8(int64_t rows, int64_t cols, const uint8_t *d_bitmap,
                                                 const uint8_t *d_values, int64_t nnz,
                                                 const int64_t *d_row_offsets, const int64_t *d_sel,
                                                 int64_t nsel, uint8_t *d_out, void *stream) {
    return run_cols(1, rows, cols, d_bitmap, d_values, nnz, d_row_offsets, d_sel, nsel, d_out, stream);
}
