// Fused small-batch product on the compressed form, on the matrix cores of gfx950:
//     Y[b][i] = sum_j W[i][j] * X[b][j],   b < nb <= 16,
// with W in the Endor bitmap format (Section 4.1) and never written out densely.  This is
// the linear operation the decompressed weight is used for (Section 3.1) for a few tokens
// at once, computed on the sparse form as Section 7 ("Efficient Compute Unit") suggests.
//
// Shape of the computation.  v_mfma_f32_16x16x32_f16 multiplies a 16 x 32 block of W (its A
// operand: lane l holds the 8 consecutive columns 8*(l/16) .. +7 of row l%16) with a 32 x 16
// block of X^T (B operand: lane l holds the same 8 columns of right-hand side l%16) into a
// 16 x 16 fp32 tile.  So one wave owns 16 rows of W and walks them 256 columns at a time
// (4096 elements per round, 8 matrix instructions); the 16 bytes an expander lane produces
// per step are exactly one lane's A operand, and the expansion is shared by all nb
// right-hand sides.
//
// A round, for the lane that is (row r = l/4, word j = l%4) while loading and
// (row l%16, column block l/16) while multiplying:
//   1. load the lane's 64 bitmap bits of the segment; popcount; prefix over the row's four
//      words (DPP quad broadcasts).  Each row has its own cursor into `values` (its 1 bits
//      so far), so the 16 rows are 16 independent streams.
//   2. load the rows' value slices for the segment: 16-byte units from the 16-byte boundary
//      below each cursor.  For this the lanes regroup as eight per row (rows l/8 and 8 + l/8),
//      so that a load instruction fetches whole 128-byte lines (with four lanes per row and
//      64-byte pieces the counters showed 1.4 times the bytes fetched); five rounds cover the
//      worst case of 256 values.  Guarded so that nothing outside values[0, nnz) is read.  The
//      units go to the rows' staging areas in LDS.
//   3. per bitmap byte, one table entry: (offset of the byte's first value in the staging
//      area) << 8 | the byte.
//   4. eight steps: read the entry of (row, byte), look the byte up in a table built once
//      per wave (the rank of every bit inside the byte), gather the 8 candidate values with
//      2-byte LDS reads, merge-and-mask them with 4 v_perm_b32 whose selectors are formed from
//      the bits, and issue the matrix instruction against the 16-byte fragment of X.
// The loads of round t+1 (bitmap, values, X) are issued before the steps of round t, so a
// wave keeps memory traffic in flight while it multiplies.
//
// Work is split over rows (16 per wave) and, to have enough waves, over column ranges
// (ksplit ranges per row group); the starting cursor of a row at a column range comes from
// the tile offset table (rank of an arbitrary position = chunk start + tile offset +
// popcount of the tile's words below it).  Partial sums of the column ranges go to a scratch
// buffer and are added in a fixed order by a second kernel, so results are reproducible.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "endor.h"
#include "endor_device.h"
#include "endor_layout.h"

namespace {

using endor_device::chunk_base;
using endor_device::u32x4;
using endor_device::wave_sum;
using endor_layout::chunks_of;
using endor_layout::chunk_total_bytes;
using endor_layout::dims_ok;
using endor_layout::kChunkStride;
using endor_layout::kTileElems;
using endor_layout::kTilesPerChunk;
using endor_layout::kTileWords;
using endor_layout::workspace_bytes_n;

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kRows = 16;               // rows of W per wave: the M of the matrix instruction
constexpr int kSegCols = 256;           // columns per round
constexpr int kSteps = kSegCols / 32;   // matrix instructions per round
constexpr int kRounds = 5;              // rounds of value loads per half of the rows: 8 lanes x 5 units >= 33
constexpr int kRowUnits = 8 * kRounds;  // staging units per row
constexpr int kInfoStride = 36;         // dwords per row of the entry table (32 used; 36 spreads the LDS banks)
constexpr int kMaxSplit = 16;           // column ranges per row group at most

struct GemmParams {
    const uint64_t *bitmap;
    const uint16_t *values;
    const uint32_t *chunk_total;
    const uint32_t *tile_off;
    const uint16_t *x;  // nb right-hand sides of cols fp16 values, ldx elements apart
    float *out;         // ksplit == 1: y (nb x rows); else the scratch: ksplit x nb x rows partial sums
    int64_t rows, cols, nnz, ldx;
    int32_t nb;
    uint32_t ksplit;
    uint32_t segs_per_split;  // rounds per column range
    uint32_t x_fast;          // every fragment of X is a 16-byte aligned, in-range load
};

// Staging rows are 584 bytes apart, not 576: the 16 rows advance through their slices in
// step, so with a pitch that is a multiple of 64 bytes (half the LDS banks) the 2-byte gathers of the
// 16 rows would pile onto the same few banks; 146 dwords (= 18 mod 32) put the rows on 16
// different even banks.  The price: units are written as two 8-byte stores.
constexpr int kRowPitch8 = 2 * kRowUnits + 1;  // 64-bit words per staging row

struct alignas(16) GemmScratch {
    uint64_t rank2[256];                // byte pattern -> 2 * (number of lower 1 bits), one byte per bit
    uint64_t stage[kRows][kRowPitch8];  // the rows' value slices of the current segment
    uint32_t info[kRows][kInfoStride];  // per (row, bitmap byte): staging offset of its first value << 8 | byte
};

// value of lane `k` of each group of four lanes, in all four
template <int k>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t x) {
    return static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(x), k * 0x55, 0xf, 0xf, false));
}

// 16 bytes of `values` at byte address p, with bytes outside [vbeg, vend) read as 0
__device__ __forceinline__ u32x4 load_values16(uintptr_t p, uintptr_t vbeg, uintptr_t vend) {
    if (p >= vbeg && p + 16 <= vend) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    uint32_t d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uintptr_t q = p + 2 * j;
        uint32_t v = 0;
        if (q >= vbeg && q + 2 <= vend) v = *reinterpret_cast<const uint16_t *>(q);
        d[j >> 1] |= v << (16 * (j & 1));
    }
    u32x4 r;
    r.x = d[0];
    r.y = d[1];
    r.z = d[2];
    r.w = d[3];
    return r;
}

// 64 bits of the bitmap starting at bit position e, of which the first nbits (0..64) count
__device__ __forceinline__ uint64_t bits_at(const uint64_t *bitmap, int64_t nwords, int64_t e, int64_t nbits) {
    if (nbits <= 0) return 0;
    const int64_t w0 = e >> 6;
    const uint32_t bs = static_cast<uint32_t>(e & 63);
    uint64_t word = (w0 < nwords ? bitmap[w0] : 0) >> bs;
    if (bs != 0) word |= (w0 + 1 < nwords ? bitmap[w0 + 1] : 0) << (64 - bs);
    if (nbits < 64) word &= (uint64_t(1) << nbits) - 1;
    return word;
}

// what a lane has in flight for the coming round
struct Round {
    uint64_t word;      // the lane's 64 bitmap bits (row l/4, word l%4 of the segment)
    u32x4 va[kRounds];  // units of the value slice of row l/8 ...
    u32x4 vb[kRounds];  // ... and of row 8 + l/8 (value-loading role: unit q*8 + l%8 in round q)
    uint32_t na, nb;    // units those two rows' slices span
    uint32_t first2;    // 2 * (staging index of the first value of the lane's word)
    u32x4 xb[kSteps];   // fragments of X (as multiplying lane: right-hand side l%16, column block l/16)
};

__global__ __launch_bounds__(64) void endor_gemm_f16_kernel(GemmParams G) {
    __shared__ GemmScratch S;
    const uint32_t lane = threadIdx.x;
    const uint32_t group = blockIdx.x / G.ksplit;  // 16 rows
    const uint32_t split = blockIdx.x % G.ksplit;  // column range
    const int64_t row0 = int64_t(group) * kRows;
    const int64_t n = G.rows * G.cols;
    const int64_t nwords = (n + 63) >> 6;
    const int64_t total_segs = (G.cols + kSegCols - 1) / kSegCols;
    const int64_t seg_begin = int64_t(split) * G.segs_per_split;
    int64_t seg_end = seg_begin + G.segs_per_split;
    if (seg_end > total_segs) seg_end = total_segs;
    const int64_t c_begin = seg_begin * kSegCols;

    // ---- the rank table, four byte patterns per lane
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const uint32_t pat = t * 64 + lane;
        uint64_t rk = 0;
        uint32_t below = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            rk |= uint64_t(2 * below) << (8 * j);
            below += (pat >> j) & 1;
        }
        S.rank2[pat] = rk;
    }

    // ---- loading role: row lr = lane/4, word lj = lane%4 of a segment
    const uint32_t lr = lane >> 2, lj = lane & 3;
    const int64_t my_row = row0 + lr;
    const bool row_ok = my_row < G.rows;
    const uintptr_t vbeg = reinterpret_cast<uintptr_t>(G.values);
    const uintptr_t vend = vbeg + 2 * static_cast<uintptr_t>(G.nnz);

    // Cursor of every row at the first column of the range: the number of 1 bits before flat
    // position e_r = row*cols + c_begin is (start of its chunk) + (tile offset) + (1 bits of
    // the tile's words below e_r).  Lane r < 16 looks up the first two terms of row r, the
    // whole wave counts the third for each row in turn; all loads go out before the first
    // result is needed, so the 16 lookups cost one trip to memory, not sixteen.
    uintptr_t cursor = vbeg;
    if (c_begin < G.cols) {  // wave-uniform
        const int64_t e_first = row0 * G.cols + c_begin;
        const uint32_t c_first = static_cast<uint32_t>(e_first >> 20);  // chunk = 2^20 positions
        int64_t last_row = row0 + kRows - 1;
        if (last_row >= G.rows) last_row = G.rows - 1;
        const uint32_t span = static_cast<uint32_t>((last_row * G.cols + c_begin) >> 20) - c_first;  // chunks after the first
        // totals of the chunks the 16 rows start in, scanned: lane k holds sum of chunks c_first .. c_first+k
        uint32_t incl = 0;
        uint64_t wide = 0;  // the same for rows so wide that the 16 starts span more than 64 chunks
        if (span <= 64) {
            const uint32_t ct = lane < span ? G.chunk_total[c_first + lane] : 0u;
            incl = endor_device::wave_inclusive_scan(ct);  // < 2^26
        }
        const uint64_t cb0 = chunk_base(G.chunk_total, c_first, lane);
        // per-row part, lane r for row r
        uint64_t head = 0;  // chunk start + tile offset of row `lane`
        {
            const int64_t row = row0 + (lane & 15);
            const int64_t e = (row < G.rows ? row : last_row) * G.cols + c_begin;
            const uint32_t c = static_cast<uint32_t>(e >> 20);
            const uint32_t k = c - c_first;  // <= span
            uint32_t before_chunk = static_cast<uint32_t>(
                __builtin_amdgcn_ds_bpermute(static_cast<int>(4 * (k ? k - 1 : 0)), static_cast<int>(incl)));
            if (k == 0) before_chunk = 0;
            if (span > 64) {
                for (uint32_t j = c_first; j < c; ++j) wide += G.chunk_total[j];
                before_chunk = 0;
            }
            const uint32_t tl = static_cast<uint32_t>((e >> 12) % kTilesPerChunk);
            head = cb0 + wide + before_chunk + G.tile_off[size_t(c) * kChunkStride + tl];
        }
        // the tile's words below e_r, for each row
        uint64_t words[kRows];
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const int64_t row = row0 + r < G.rows ? row0 + r : last_row;
            const int64_t e = row * G.cols + c_begin;
            const int64_t w = (e >> 12) * kTileWords + lane, we = e >> 6;
            uint64_t word = 0;
            if (w <= we) word = G.bitmap[w];  // w <= we < number of words
            if (w == we) word &= (uint64_t(1) << (e & 63)) - 1;
            words[r] = word;
        }
        uint32_t below = 0;  // lane r: 1 bits of row r's tile below e_r
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const uint32_t sum = wave_sum(__popcll(words[r]));
            if (lane == static_cast<uint32_t>(r)) below = sum;
        }
        const uint64_t rank = head + below;  // lane r < 16: row r
        const uint32_t lo = static_cast<uint32_t>(
            __builtin_amdgcn_ds_bpermute(static_cast<int>(4 * lr), static_cast<int>(static_cast<uint32_t>(rank))));
        const uint32_t hi = static_cast<uint32_t>(
            __builtin_amdgcn_ds_bpermute(static_cast<int>(4 * lr), static_cast<int>(static_cast<uint32_t>(rank >> 32))));
        cursor = vbeg + 2 * ((uint64_t(hi) << 32) | lo);
    }

    // ---- multiplying role: row mr = lane%16 (A) / right-hand side mr (B), column block mq = lane/16
    const uint32_t mr = lane & 15, mq = lane >> 4;
    const uint16_t *xrow = G.x + int64_t(mr) * G.ldx;
    const bool x_ok = static_cast<int32_t>(mr) < G.nb;

    // Shapes whose rows start on 64-bit word boundaries (cols a multiple of 64: every model
    // shape) read a lane's bitmap word with one aligned load; others funnel it out of two.
    const bool word_rows = (G.cols & 63) == 0;  // wave-uniform
    const uint64_t *my_words = G.bitmap + ((row_ok ? my_row : 0) * G.cols >> 6) + lj;
    const uint16_t *x_lane = xrow + 8 * mq;

    auto issue = [&](int64_t seg, Round &R) {
        const int64_t c0 = seg * kSegCols;
        const int64_t col = c0 + 64 * lj;
        if (word_rows)
            R.word = (row_ok && col < G.cols) ? my_words[c0 >> 6] : 0;
        else
            R.word = row_ok ? bits_at(G.bitmap, nwords, my_row * G.cols + col, G.cols - col) : 0;
        const uint32_t pc = __popcll(R.word);
        const uint32_t p0 = quad_bcast<0>(pc), p1 = quad_bcast<1>(pc), p2 = quad_bcast<2>(pc), p3 = quad_bcast<3>(pc);
        const uint32_t before = (lj > 0 ? p0 : 0) + (lj > 1 ? p1 : 0) + (lj > 2 ? p2 : 0);
        const uint32_t cnt = p0 + p1 + p2 + p3;  // <= 256
        const uintptr_t a16 = cursor & ~uintptr_t(15);
        const uint32_t shift = static_cast<uint32_t>(cursor - a16) >> 1;  // values of slack in front
        const uint32_t nunits = cnt ? ((shift + cnt) * 2 + 15) >> 4 : 0;  // <= 33
        R.first2 = 2 * (shift + before);
        // a row slice that lies inside values[0, nnz) with its rounding to 16-byte units (all but
        // the first and last few values of the array) needs no per-unit range checks
        const bool inside = a16 >= vbeg && a16 + 16 * uintptr_t(nunits) <= vend;
        const bool all_inside = __builtin_amdgcn_ballot_w64(!inside) == 0;  // wave-uniform
        // Value-loading role: eight lanes per row, so that one load instruction fetches whole
        // 128-byte lines (rows l/8 and 8 + l/8; their slice start and length come from the
        // lanes that own the rows' cursors).
        const uint32_t a_lo = static_cast<uint32_t>(a16), a_hi = static_cast<uint32_t>(a16 >> 32);
        const int own_a = static_cast<int>(16 * (lane >> 3)), own_b = own_a + 128;  // byte index of lane 4*row
        const uintptr_t base_a = (uintptr_t(static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(own_a, a_hi))) << 32) |
                                 static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(own_a, a_lo));
        const uintptr_t base_b = (uintptr_t(static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(own_b, a_hi))) << 32) |
                                 static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(own_b, a_lo));
        R.na = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(own_a, static_cast<int>(nunits)));
        R.nb = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(own_b, static_cast<int>(nunits)));
        const uint32_t sub = lane & 7;
        if (all_inside) {
            const u32x4 *pa = reinterpret_cast<const u32x4 *>(base_a) + sub;
            const u32x4 *pb = reinterpret_cast<const u32x4 *>(base_b) + sub;
#pragma unroll
            for (int q = 0; q < kRounds; ++q) {
                if (uint32_t(q * 8) + sub < R.na) R.va[q] = __builtin_nontemporal_load(pa + q * 8);
                if (uint32_t(q * 8) + sub < R.nb) R.vb[q] = __builtin_nontemporal_load(pb + q * 8);
            }
        } else {
#pragma unroll
            for (int q = 0; q < kRounds; ++q) {
                const uint32_t u = q * 8 + sub;
                if (u < R.na) R.va[q] = load_values16(base_a + 16 * uintptr_t(u), vbeg, vend);
                if (u < R.nb) R.vb[q] = load_values16(base_b + 16 * uintptr_t(u), vbeg, vend);
            }
        }
        cursor += 2 * uintptr_t(cnt);
        if (G.x_fast && c0 + kSegCols <= G.cols) {  // wave-uniform: every fragment is a whole aligned load
#pragma unroll
            for (int t = 0; t < kSteps; ++t) {
                u32x4 f;
                f.x = f.y = f.z = f.w = 0;
                if (x_ok) f = *reinterpret_cast<const u32x4 *>(x_lane + c0 + 32 * t);
                R.xb[t] = f;
            }
        } else {
#pragma unroll
            for (int t = 0; t < kSteps; ++t) {
                const int64_t c = c0 + 32 * t + 8 * mq;
                uint32_t h[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) h[j] = (x_ok && c + j < G.cols) ? uint32_t(xrow[c + j]) : 0u;
                u32x4 f;
                f.x = h[0] | (h[1] << 16);
                f.y = h[2] | (h[3] << 16);
                f.z = h[4] | (h[5] << 16);
                f.w = h[6] | (h[7] << 16);
                R.xb[t] = f;
            }
        }
    };

    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    Round R;
    if (seg_begin < seg_end) issue(seg_begin, R);
    for (int64_t seg = seg_begin; seg < seg_end; ++seg) {
        // ---- land the round's loads in LDS: entries of the lane's 8 bitmap bytes, value units
        {
            uint32_t e8[8];
            uint32_t at2 = R.first2;
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const uint32_t byte = static_cast<uint32_t>(R.word >> (8 * b)) & 0xffu;
                e8[b] = (at2 << 8) | byte;
                at2 += 2 * __popc(byte);
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
            u32x4 *ip = reinterpret_cast<u32x4 *>(&S.info[lr][lj * 8]);
            ip[0] = lo;
            ip[1] = hi;
            const uint32_t ra = lane >> 3, sub = lane & 7;
#pragma unroll
            for (int q = 0; q < kRounds; ++q) {
                const uint32_t u = q * 8 + sub;
                if (u < R.na) {
                    S.stage[ra][2 * u] = uint64_t(R.va[q].x) | (uint64_t(R.va[q].y) << 32);
                    S.stage[ra][2 * u + 1] = uint64_t(R.va[q].z) | (uint64_t(R.va[q].w) << 32);
                }
                if (u < R.nb) {
                    S.stage[ra + 8][2 * u] = uint64_t(R.vb[q].x) | (uint64_t(R.vb[q].y) << 32);
                    S.stage[ra + 8][2 * u + 1] = uint64_t(R.vb[q].z) | (uint64_t(R.vb[q].w) << 32);
                }
            }
        }
        // This round's fragments of X must have arrived before the next round's loads are
        // issued: the hardware counts outstanding loads in order, so a wait placed after the
        // new loads would wait for them as well.  The empty asm makes the values "used" here.
        u32x4 xb[kSteps];
#pragma unroll
        for (int t = 0; t < kSteps; ++t) {
            xb[t] = R.xb[t];
            asm volatile("" : "+v"(xb[t].x), "+v"(xb[t].y), "+v"(xb[t].z), "+v"(xb[t].w));
        }
        // LDS operations of one wave execute in issue order; the fences only pin the compiler
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- next round's loads go out before this round's arithmetic
        if (seg + 1 < seg_end) issue(seg + 1, R);

        // ---- 8 steps: expand 8 elements of row mr, multiply.  The table reads of all steps go
        //      out first, then the gathers two steps at a time, so that the LDS latencies of
        //      different steps overlap.
        const uint8_t *row_stage = reinterpret_cast<const uint8_t *>(&S.stage[mr][0]);
        uint32_t entry[kSteps];
        uint64_t rk[kSteps];
#pragma unroll
        for (int t = 0; t < kSteps; ++t) entry[t] = S.info[mr][t * 4 + mq];
#pragma unroll
        for (int t = 0; t < kSteps; ++t) rk[t] = S.rank2[entry[t] & 0xffu];
#pragma unroll
        for (int t0 = 0; t0 < kSteps; t0 += 2) {
            uint32_t h[2][8];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint8_t *base = row_stage + (entry[t0 + u] >> 8);
                const uint32_t rlo = static_cast<uint32_t>(rk[t0 + u]), rhi = static_cast<uint32_t>(rk[t0 + u] >> 32);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    h[u][j] = *reinterpret_cast<const uint16_t *>(base + ((rlo >> (8 * j)) & 0xffu));
                    h[u][4 + j] = *reinterpret_cast<const uint16_t *>(base + ((rhi >> (8 * j)) & 0xffu));
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint32_t bits = entry[t0 + u] & 0xffu;
                // v_perm_b32(hi, lo, sel): selector bytes 0,1 take lo's low half, 4,5 hi's low half
                // and 0x0c gives 0, so sel = 0x0c0c0c0c with 0x0100 / 0x0504 put in where the bit
                // is 1: XOR with 0x0d0c (low half) and 0x0908 (high half) under the sign-extended bits
                uint32_t a4[4];
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const uint32_t m0 = static_cast<uint32_t>(static_cast<int32_t>(bits << (31 - 2 * d)) >> 31);
                    const uint32_t m1 = static_cast<uint32_t>(static_cast<int32_t>(bits << (30 - 2 * d)) >> 31);
                    const uint32_t sel = 0x0c0c0c0cu ^ (m0 & 0x00000d0cu) ^ (m1 & 0x09080000u);
                    a4[d] = __builtin_amdgcn_perm(h[u][2 * d + 1], h[u][2 * d], sel);
                }
                u32x4 a;
                a.x = a4[0];
                a.y = a4[1];
                a.z = a4[2];
                a.w = a4[3];
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                             __builtin_bit_cast(f16x8, xb[t0 + u]), acc, 0, 0, 0);
            }
        }
        // the next round's LDS writes must stay behind this round's LDS reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    // ---- lane l holds rows 4*(l/16) .. +3 of right-hand side l%16
    if (x_ok) {
        float *dst = G.out + (size_t(split) * G.nb + mr) * G.rows + row0 + 4 * mq;
        const float a4[4] = {acc[0], acc[1], acc[2], acc[3]};
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (row0 + 4 * mq + i < G.rows) dst[i] = a4[i];
    }
}

// y[b][i] = sum over the column ranges, in ascending order
__global__ __launch_bounds__(256) void endor_gemm_reduce_kernel(const float *__restrict__ partial, float *__restrict__ y,
                                                                int64_t count, uint32_t ksplit) {
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= count) return;
    float s = partial[i];
    for (uint32_t k = 1; k < ksplit; ++k) s += partial[size_t(k) * count + i];
    y[i] = s;
}

__global__ __launch_bounds__(256) void endor_gemm_zero_kernel(float *__restrict__ y, int64_t count) {
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (i < count) y[i] = 0.0f;
}

// column ranges per row group: enough waves to fill the chip, never more than kMaxSplit
uint32_t choose_split(int64_t rows, int64_t cols) {
    const int64_t groups = (rows + kRows - 1) / kRows;
    const int64_t segs = (cols + kSegCols - 1) / kSegCols;
    int64_t k = (6144 + groups - 1) / groups;  // about 24 waves per compute unit
    if (k > kMaxSplit) k = kMaxSplit;
    if (k > segs) k = segs;
    if (k < 1) k = 1;
    return static_cast<uint32_t>(k);
}

}  // namespace

extern "C" size_t endor_gemm_scratch_bytes(int64_t rows, int64_t cols, int nb) {
    if (!dims_ok(rows, cols) || nb < 1 || nb > ENDOR_GEMM_MAX_BATCH || rows == 0 || cols == 0) return 0;
    const uint32_t ksplit = choose_split(rows, cols);
    if (ksplit == 1) return 0;
    return (static_cast<size_t>(ksplit) * nb * rows * sizeof(float) + 255) & ~size_t(255);
}

extern "C" endor_status endor_gemm_f16(int64_t rows, int64_t cols, const uint8_t *d_bitmap, const uint16_t *d_values,
                                       int64_t nnz, const void *d_workspace, size_t workspace_bytes,
                                       const uint16_t *d_x, int64_t ldx, int nb, float *d_y, void *d_scratch,
                                       size_t scratch_bytes, void *stream) {
    if (rows < 0 || cols < 0 || nnz < 0 || nb < 0 || nb > ENDOR_GEMM_MAX_BATCH) return ENDOR_ERR_INVALID_ARG;
    if (!dims_ok(rows, cols)) return ENDOR_ERR_UNSUPPORTED;
    if (rows == 0 || nb == 0) return ENDOR_OK;
    if (rows > (int64_t(1) << 31) - kRows) return ENDOR_ERR_UNSUPPORTED;
    if (!d_y || (reinterpret_cast<uintptr_t>(d_y) & 3)) return ENDOR_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t count = int64_t(nb) * rows;
    if (cols == 0) {
        // an empty sum: every output is +0.0 (a fill kernel, so that the call can be captured into a graph)
        hipLaunchKernelGGL(endor_gemm_zero_kernel, dim3(static_cast<unsigned>((count + 255) / 256)), dim3(256), 0, s, d_y,
                           count);
        return hipGetLastError() == hipSuccess ? ENDOR_OK : ENDOR_ERR_HIP;
    }
    if (nnz > rows * cols || ldx < cols) return ENDOR_ERR_INVALID_ARG;
    if (!d_bitmap || (reinterpret_cast<uintptr_t>(d_bitmap) & 7)) return ENDOR_ERR_INVALID_ARG;
    if (!d_x || (reinterpret_cast<uintptr_t>(d_x) & 1)) return ENDOR_ERR_INVALID_ARG;
    if (nnz > 0 && (!d_values || (reinterpret_cast<uintptr_t>(d_values) & 1))) return ENDOR_ERR_INVALID_ARG;
    const int64_t n = rows * cols;
    if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 255)) return ENDOR_ERR_INVALID_ARG;
    if (workspace_bytes < workspace_bytes_n(n)) return ENDOR_ERR_BUFFER_TOO_SMALL;
    const uint32_t ksplit = choose_split(rows, cols);
    const size_t need = endor_gemm_scratch_bytes(rows, cols, nb);
    if (ksplit > 1) {
        if (!d_scratch || (reinterpret_cast<uintptr_t>(d_scratch) & 255)) return ENDOR_ERR_INVALID_ARG;
        if (scratch_bytes < need) return ENDOR_ERR_BUFFER_TOO_SMALL;
    }
    GemmParams G;
    G.bitmap = reinterpret_cast<const uint64_t *>(d_bitmap);
    G.values = d_values;
    G.chunk_total = static_cast<const uint32_t *>(d_workspace);
    G.tile_off = reinterpret_cast<const uint32_t *>(static_cast<const char *>(d_workspace) + chunk_total_bytes(n));
    G.x = d_x;
    G.out = ksplit == 1 ? d_y : static_cast<float *>(d_scratch);
    G.rows = rows;
    G.cols = cols;
    G.nnz = nnz;
    G.ldx = ldx;
    G.nb = nb;
    G.ksplit = ksplit;
    const int64_t segs = (cols + kSegCols - 1) / kSegCols;
    G.segs_per_split = static_cast<uint32_t>((segs + ksplit - 1) / ksplit);
    G.x_fast = ((reinterpret_cast<uintptr_t>(d_x) & 15) == 0 && (ldx * 2) % 16 == 0) ? 1u : 0u;
    const int64_t groups = (rows + kRows - 1) / kRows;
    hipLaunchKernelGGL(endor_gemm_f16_kernel, dim3(static_cast<unsigned>(groups * ksplit)), dim3(64), 0, s, G);
    if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
    if (ksplit > 1) {
        hipLaunchKernelGGL(endor_gemm_reduce_kernel, dim3(static_cast<unsigned>((count + 255) / 256)), dim3(256), 0, s,
                           static_cast<const float *>(d_scratch), d_y, count, ksplit);
        if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
    }
    return ENDOR_OK;
}
