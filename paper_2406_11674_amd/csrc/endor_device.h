// Wave-level building blocks shared by the device code of the Endor library (gfx950, wave64):
// prefix sums across the lanes of a wave with DPP row shifts and broadcasts, and the lookup of
// a chunk's absolute start from the per-chunk totals of the offset table.
#ifndef ENDOR_DEVICE_H_
#define ENDOR_DEVICE_H_

#include <hip/hip_runtime.h>

#include <cstdint>

namespace endor_device {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int kCtrl, int kRowMask>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t x) {
    // lanes without a source, and rows masked off, receive 0
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), kCtrl, kRowMask, 0xf, true));
}

// inclusive prefix sum within each row of 16 lanes (row_shr:1,2,4,8)
__device__ __forceinline__ uint32_t row_inclusive_scan(uint32_t x) {
    x += dpp_or_zero<0x111, 0xf>(x);
    x += dpp_or_zero<0x112, 0xf>(x);
    x += dpp_or_zero<0x114, 0xf>(x);
    x += dpp_or_zero<0x118, 0xf>(x);
    return x;
}

// inclusive prefix sum over the 64 lanes of a wave
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x) {
    x = row_inclusive_scan(x);
    x += dpp_or_zero<0x142, 0xa>(x);  // row_bcast:15 into rows 1 and 3
    x += dpp_or_zero<0x143, 0xc>(x);  // row_bcast:31 into rows 2 and 3
    return x;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t x) {
    return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(wave_inclusive_scan(x)), 63));
}

// Number of 1 bits before chunk c of the matrix: sum of the earlier chunks' totals.
// c < 2^14 and a total is at most 2^20, so a lane's partial sum fits 32 bits; the
// two 16-bit halves are summed across lanes separately to keep 64 bits.
__device__ __forceinline__ uint64_t chunk_base(const uint32_t *chunk_total, uint32_t c, uint32_t lane) {
    if (c == 0) return 0;
    uint32_t part = 0;
    for (uint32_t j = lane; j < c; j += 64) part += chunk_total[j];
    const uint32_t lo = wave_sum(part & 0xffffu);
    const uint32_t hi = wave_sum(part >> 16);
    return uint64_t(lo) + (uint64_t(hi) << 16);
}

}  // namespace endor_device

#endif  // ENDOR_DEVICE_H_
