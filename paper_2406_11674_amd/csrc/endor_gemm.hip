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
//   1. the lane's 64 bitmap bits of the segment (loaded a round ahead); popcount; prefix over
//      the row's four words (DPP quad broadcasts).  Each row has its own cursor into `values`
//      (its 1 bits so far), so the 16 rows are 16 independent streams.
//   2. per bitmap byte, one table entry in LDS: (values of the row's segment before the byte)
//      << 8 | the byte.
//   3. eight steps: read the entry of (row, byte), read the byte's window of values (16 bytes
//      from the row's cursor plus the entry's count) straight from memory, move the values to
//      the positions of the 1 bits with v_perm_b32 (selectors from a table indexed by the
//      byte), and issue the matrix instruction against the 16-byte fragment of X.
// Values are not staged: the windows of a row's neighbouring bytes overlap and the vector
// cache serves the overlap.  The expansion runs in the loading role's lane order, where the
// four lanes of a quad read neighbouring windows of one row, and the expanded 16 bytes are
// handed to the multiplying lane with ds_bpermute.  (An earlier form staged every row's slice
// in LDS and gathered the values one by one: 126 / 138 us for 1 / 16 right-hand sides on
// 28672 x 8192, bound by LDS; this one takes 91 / 101 us, bound by the rate at which the
// vector cache accepts line accesses.)  A round's eight window loads per lane go out back to
// back behind one wave-uniform bounds test; the rounds at the very ends of `values` take a
// rolled loop with guarded element-wise loads instead.
// X: the four waves of a workgroup work on neighbouring row groups and the same column
// range; the round's 256 columns of all right-hand sides are brought to LDS once per
// workgroup (global_load_lds_dwordx4, double buffered, one barrier per round) and every wave
// reads its B operands from there.
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
using endor_device::load_to_lds16;
using endor_device::window_finish;
using endor_device::window_guarded;
using endor_device::window_issue;
using endor_device::WindowLoad;
using endor_device::windows_inside;
using endor_device::place_window;
using endor_device::window_tables_init;
using endor_device::WindowTables;
using endor_device::u32x4;
using endor_device::wait_loads_to_lds;
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
constexpr int kInfoStride = 36;         // dwords per row of the entry table (32 used; 36 spreads the LDS banks)
constexpr int kMaxSplit = 16;           // column ranges per row group at most
constexpr int kGemmWaves = 4;           // waves (row groups) per workgroup; they share the tile of X
constexpr int kXPitch = 2 * kSegCols + 16;  // bytes between right-hand sides in the LDS tile of X: 132 dwords, so the
                                            // 16-byte reads of eight lanes (eight right-hand sides) cover all 32 banks

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

struct alignas(16) GemmScratch {
    WindowTables tables;  // selectors of the value placement, per byte pattern
    // per wave and (row, bitmap byte): values of the row's segment before it << 8 | byte
    uint32_t info[kGemmWaves][kRows][kInfoStride];
    // the segment's 256 columns of the 16 right-hand sides, for this round and the next
    alignas(16) uint8_t xt[2][ENDOR_GEMM_MAX_BATCH][kXPitch];
};

// value of lane `k` of each group of four lanes, in all four
template <int k>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t x) {
    return static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(x), k * 0x55, 0xf, 0xf, false));
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

__global__ __launch_bounds__(64 * kGemmWaves) void endor_gemm_f16_kernel(GemmParams G) {
    __shared__ GemmScratch S;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // a workgroup: kGemmWaves neighbouring groups of 16 rows, one column range.  A group past
    // the last row still runs (with no valid row): its wave takes part in loading X.
    const uint32_t group = (blockIdx.x / G.ksplit) * kGemmWaves + wave;
    const uint32_t split = blockIdx.x % G.ksplit;
    const int64_t row0 = int64_t(group) * kRows;
    const int64_t n = G.rows * G.cols;
    const int64_t nwords = (n + 63) >> 6;
    const int64_t total_segs = (G.cols + kSegCols - 1) / kSegCols;
    const int64_t seg_begin = int64_t(split) * G.segs_per_split;
    int64_t seg_end = seg_begin + G.segs_per_split;
    if (seg_end > total_segs) seg_end = total_segs;
    const int64_t c_begin = seg_begin * kSegCols;

    window_tables_init(S.tables, threadIdx.x);  // visible after the first round's barrier
    uint32_t(*info)[kInfoStride] = S.info[wave];

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
    if (c_begin < G.cols && row0 < G.rows) {  // wave-uniform
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
    const bool x_ok = static_cast<int32_t>(mr) < G.nb;

    // Shapes whose rows start on 64-bit word boundaries (cols a multiple of 64: every model
    // shape) read a lane's bitmap word with one aligned load; others funnel it out of two.
    const bool word_rows = (G.cols & 63) == 0;  // wave-uniform
    const uint64_t *my_words = G.bitmap + ((row_ok ? my_row : 0) * G.cols >> 6) + lj;

    // this lane's 64 bitmap bits of a segment (loading role)
    auto load_word = [&](int64_t seg) -> uint64_t {
        const int64_t col = seg * kSegCols + 64 * lj;
        if (word_rows) return (row_ok && col < G.cols) ? my_words[(seg * kSegCols) >> 6] : 0;
        return row_ok ? bits_at(G.bitmap, nwords, my_row * G.cols + col, G.cols - col) : 0;
    };

    // Expansion happens in the loading role (a quad of lanes = four neighbouring bytes of one
    // row, whose windows share cache lines; with the multiplying role's lane order every lane
    // of a load would touch a line of its own, and the vector cache's access rate was the
    // bound: 1400 accesses per round against 400).  The expanded 16 bytes then move to the lane
    // that multiplies them: lane 16*j + r takes those of lane 4*r + j.
    const int from_lane = static_cast<int>(4 * (4 * mr + mq));  // byte index for ds_bpermute

    // The segment's 256 columns of X go to LDS once per workgroup: wave w brings the right-hand
    // sides 4w .. 4w+3 (those below nb), 512 bytes each, with the first 32 lanes.
    auto load_x_tile = [&](int64_t seg, uint32_t buf) {
        const int64_t c0 = seg * kSegCols;
        const bool whole = G.x_fast && c0 + kSegCols <= G.cols;  // aligned 16-byte pieces, all in range
#pragma unroll
        for (int i = 0; i < ENDOR_GEMM_MAX_BATCH / kGemmWaves; ++i) {
            const int b = static_cast<int>(wave) * (ENDOR_GEMM_MAX_BATCH / kGemmWaves) + i;
            if (b < G.nb && lane < 32) {
                const uint16_t *src = G.x + int64_t(b) * G.ldx + c0;
                u32x4 *dst = reinterpret_cast<u32x4 *>(S.xt[buf][b]);
                if (whole) {
                    load_to_lds16<false>(reinterpret_cast<const u32x4 *>(src) + lane, dst);
                } else {
                    uint32_t h[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) h[j] = (c0 + 8 * lane + j < G.cols) ? uint32_t(src[8 * lane + j]) : 0u;
                    u32x4 f;
                    f.x = h[0] | (h[1] << 16);
                    f.y = h[2] | (h[3] << 16);
                    f.z = h[4] | (h[5] << 16);
                    f.w = h[6] | (h[7] << 16);
                    dst[lane] = f;
                }
            }
        }
    };

    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    if (seg_begin < seg_end) load_x_tile(seg_begin, 0);
    uint64_t word = seg_begin < seg_end ? load_word(seg_begin) : 0;
    for (int64_t seg = seg_begin; seg < seg_end; ++seg) {
        const uint32_t buf = static_cast<uint32_t>(seg - seg_begin) & 1u;
        // this wave's part of the round's tile of X has landed; after the barrier the whole tile
        // has, and every wave is through the previous round (whose tile the next load overwrites)
        wait_loads_to_lds();
        __syncthreads();
        if (seg + 1 < seg_end) load_x_tile(seg + 1, buf ^ 1u);
        // ---- entries of the lane's 8 bitmap bytes
        const uint32_t pc = __popcll(word);
        const uint32_t p0 = quad_bcast<0>(pc), p1 = quad_bcast<1>(pc), p2 = quad_bcast<2>(pc), p3 = quad_bcast<3>(pc);
        const uint32_t cnt = p0 + p1 + p2 + p3;  // values of the row's segment: <= 256
        {
            uint32_t at = (lj > 0 ? p0 : 0) + (lj > 1 ? p1 : 0) + (lj > 2 ? p2 : 0);
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
            u32x4 *ip = reinterpret_cast<u32x4 *>(&info[lr][lj * 8]);
            ip[0] = lo;
            ip[1] = hi;
        }
        // LDS operations of one wave execute in issue order; the fences only pin the compiler
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- loads: the next segment's bitmap word, this segment's windows
        const uint64_t next_word = seg + 1 < seg_end ? load_word(seg + 1) : 0;
        const uint8_t *xt = &S.xt[buf][mr][16 * mq];  // right-hand side mr, column block mq of step 0
        // one step's expanded 16 bytes of row lr go to the lane that multiplies them
        auto step = [&](int t, u32x4 e) {
            u32x4 a;
            a.x = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(from_lane, static_cast<int>(e.x)));
            a.y = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(from_lane, static_cast<int>(e.y)));
            a.z = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(from_lane, static_cast<int>(e.z)));
            a.w = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(from_lane, static_cast<int>(e.w)));
            const u32x4 xb = *reinterpret_cast<const u32x4 *>(xt + 64 * t);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, xb), acc, 0,
                                                         0, 0);
        };
        // every window of this round starts in [cursor, cursor + 2 cnt] of its row; all rows' windows
        // lie inside `values` except in the rounds at the very ends of the array
        const bool row_inside = windows_inside(cursor, cursor + 2 * uintptr_t(cnt), vbeg, vend);
        if (__builtin_amdgcn_ballot_w64(!row_inside) == 0) {  // wave-uniform
            uint32_t entry[kSteps];
            WindowLoad win[kSteps];
#pragma unroll
            for (int t = 0; t < kSteps; ++t) entry[t] = info[lr][t * 4 + lj];
#pragma unroll
            for (int t = 0; t < kSteps; ++t) win[t] = window_issue(cursor + 2 * uintptr_t(entry[t] >> 8));
#pragma unroll
            for (int t = 0; t < kSteps; ++t)
                step(t, place_window(S.tables, entry[t] & 0xffu,
                                     window_finish(win[t], cursor + 2 * uintptr_t(entry[t] >> 8))));
        } else {
#pragma unroll 1
            for (int t = 0; t < kSteps; ++t) {
                const uint32_t entry = info[lr][t * 4 + lj];
                step(t, place_window(S.tables, entry & 0xffu,
                                     window_guarded(cursor + 2 * uintptr_t(entry >> 8), vbeg, vend)));
            }
        }
        // the next round's LDS writes must stay behind this round's LDS reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        cursor += 2 * uintptr_t(cnt);
        word = next_word;
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

// Column ranges per row group.  The chip holds kResident workgroups at a time (four per compute
// unit: 104 registers give four waves per SIMD, and a workgroup puts one wave on each), so the
// launch runs in ceil(workgroups / kResident) waves of workgroups, each as long as one
// workgroup: its rounds plus a start-up worth about two.  Pick the split that minimises the
// product (measured on 28672 x 8192: 4 ranges 98 us, 6 ranges, which spill into a third wave,
// 111 us; on 8192 x 28672: 8 ranges, exactly one wave of workgroups, 84 us, 10 ranges 94 us),
// the smaller one on a tie.
constexpr int64_t kResident = 256 * 4;
uint32_t choose_split(int64_t rows, int64_t cols) {
    const int64_t groups = (rows + kRows - 1) / kRows;
    const int64_t wgs = (groups + kGemmWaves - 1) / kGemmWaves;
    const int64_t segs = (cols + kSegCols - 1) / kSegCols;
    int64_t best = 1, best_cost = -1;
    for (int64_t k = 1; k <= kMaxSplit && k <= segs; ++k) {
        const int64_t per = (segs + k - 1) / k;
        if ((k - 1) * per >= segs) continue;  // the last range would be empty
        const int64_t cost = ((wgs * k + kResident - 1) / kResident) * (per + 2);
        if (best_cost < 0 || cost < best_cost) {
            best = k;
            best_cost = cost;
        }
    }
    return static_cast<uint32_t>(best);
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
    const int64_t blocks = (groups + kGemmWaves - 1) / kGemmWaves * ksplit;
    hipLaunchKernelGGL(endor_gemm_f16_kernel, dim3(static_cast<unsigned>(blocks)), dim3(64 * kGemmWaves), 0, s, G);
    if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
    if (ksplit > 1) {
        hipLaunchKernelGGL(endor_gemm_reduce_kernel, dim3(static_cast<unsigned>((count + 255) / 256)), dim3(256), 0, s,
                           static_cast<const float *>(d_scratch), d_y, count, ksplit);
        if (hipGetLastError() != hipSuccess) return ENDOR_ERR_HIP;
    }
    return ENDOR_OK;
}
