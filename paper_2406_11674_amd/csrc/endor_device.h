// Wave-level building blocks shared by the device code of the Endor library (gfx950, wave64):
// prefix sums across the lanes of a wave with DPP row shifts and broadcasts, the lookup of
// a chunk's absolute start from the per-chunk totals of the offset table, and the window
// form of the expansion used by the fused products.
#ifndef ENDOR_DEVICE_H_
#define ENDOR_DEVICE_H_

#include <hip/hip_runtime.h>

#include <cstdint>

namespace endor_device {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// A byte address known to lie in global memory, as a pointer the compiler knows to be global:
// a load through a pointer made from an integer is otherwise a FLAT instruction, which also
// counts as an LDS operation, so every wait for an LDS read waits for those loads as well.
template <class T>
__device__ __forceinline__ const __attribute__((address_space(1))) T *global_ptr(uintptr_t a) {
    return reinterpret_cast<const __attribute__((address_space(1))) T *>(a);
}
template <class T>
__device__ __forceinline__ __attribute__((address_space(1))) T *global_ptr_mut(uintptr_t a) {
    return reinterpret_cast<__attribute__((address_space(1))) T *>(a);
}

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
    // 256 totals per pass, the four loads of a lane issued together (an index past the end reads
    // the last total again and drops it: a load under a test is waited for on the spot)
    for (uint32_t j0 = 0; j0 < c; j0 += 256) {
        uint32_t t[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t j = j0 + 64 * k + lane;
            t[k] = chunk_total[j < c ? j : c - 1];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) part += (j0 + 64 * k + lane < c) ? t[k] : 0u;
    }
    const uint32_t lo = wave_sum(part & 0xffffu);
    const uint32_t hi = wave_sum(part >> 16);
    return uint64_t(lo) + (uint64_t(hi) << 16);
}

// 16 bytes per lane from global memory straight into LDS: lane l writes lds_base + 16*l
// (lds_base is wave-uniform; lanes that are switched off write nothing).  kStreamed marks the
// load non-temporal.
template <bool kStreamed = true>
__device__ __forceinline__ void load_to_lds16(const u32x4 *src, u32x4 *lds_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                     (__attribute__((address_space(3))) void *)lds_base, 16, 0, kStreamed ? 2 : 0);
}
// Every load this wave has issued is complete, those into LDS included (s_waitcnt vmcnt(0)).
__device__ __forceinline__ void wait_loads_to_lds() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// ---------------------------------------------------------------- expansion of 16-bit values, window form
//
// For the kernels that consume the expanded elements in registers (the products): the values
// a bitmap byte consumes are consecutive in `values`, at most 8 of them, so a lane reads that
// window of 16 bytes straight from memory (neighbouring lanes' windows overlap, the cache
// serves the overlap) and moves the values to their positions with v_perm_b32, whose
// selectors depend on the byte's bit pattern only and come from tables in LDS:
//     out dword 0 <- perm(w0, w0), dword 1 <- perm(w1, w0),
//     dword 2, 3  <- perm(w1, w0) | perm(w3, w2)        (w0..w3: the window, 8 halves)
// Element j of the byte takes window half popcount(bits below j); a selector byte of 0x0c
// yields zero, which also serves as the mask for 0 bits.  No staging of values in LDS and no
// per-element gathers: measured against an LDS-staged window (three two-dword LDS reads per
// byte) and against eight 2-byte LDS gathers per byte, this form is the fastest of the three.

struct alignas(16) WindowTables {
    u32x4 sel23[256];    // per byte pattern: selA, selB of output dword 2; selA, selB of dword 3
    uint64_t sel01[16];  // per low nibble: selectors of output dwords 0 and 1
};

// selector bytes that copy half k (0..3) of the 64-bit source pair {hi, lo} of a v_perm_b32
__device__ __forceinline__ uint32_t half_selector(uint32_t k) { return ((2 * k + 1) << 8) | (2 * k); }

// Fill the tables: thread t of the (at least 256-thread) workgroup writes the entry of pattern t.
__device__ __forceinline__ void window_tables_init(WindowTables &T, uint32_t t) {
    if (t < 256) {
        uint32_t sel[4] = {0x0c0c0c0cu, 0x0c0c0c0cu, 0x0c0c0c0cu, 0x0c0c0c0cu};  // A2, B2, A3, B3
#pragma unroll
        for (int e = 4; e < 8; ++e) {
            if ((t >> e) & 1) {
                const uint32_t k = __popc(t & ((1u << e) - 1));  // window half this element takes: 0..7
                const int which = 2 * ((e - 4) >> 1) + (k >= 4 ? 1 : 0);
                const uint32_t hs = half_selector(k & 3) ^ 0x0c0cu;  // XOR turns the 0x0c0c placeholder into it
                sel[which] ^= hs << (16 * (e & 1));
            }
        }
        u32x4 v;
        v.x = sel[0];
        v.y = sel[1];
        v.z = sel[2];
        v.w = sel[3];
        T.sel23[t] = v;
    }
    if (t < 16) {
        uint32_t s01[2] = {0x0c0c0c0cu, 0x0c0c0c0cu};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if ((t >> e) & 1) {
                const uint32_t k = __popc(t & ((1u << e) - 1));  // 0..3
                s01[e >> 1] ^= (half_selector(k) ^ 0x0c0cu) << (16 * (e & 1));
            }
        }
        T.sel01[t] = uint64_t(s01[0]) | (uint64_t(s01[1]) << 32);
    }
}

// The window's values moved to the positions of the 1 bits of `bits` (a bitmap byte); 0 elsewhere.
__device__ __forceinline__ u32x4 place_window(const WindowTables &T, uint32_t bits, u32x4 w) {
    const uint64_t s01 = T.sel01[bits & 15u];
    const u32x4 s23 = T.sel23[bits];
    u32x4 d;
    d.x = __builtin_amdgcn_perm(w.x, w.x, static_cast<uint32_t>(s01));
    d.y = __builtin_amdgcn_perm(w.y, w.x, static_cast<uint32_t>(s01 >> 32));
    d.z = __builtin_amdgcn_perm(w.y, w.x, s23.x) | __builtin_amdgcn_perm(w.w, w.z, s23.y);
    d.w = __builtin_amdgcn_perm(w.y, w.x, s23.z) | __builtin_amdgcn_perm(w.w, w.z, s23.w);
    return d;
}

// The 16 bytes (8 values of 16 bits) at byte address p, which is 2-byte aligned only.  Read as
// the 20 bytes from the dword boundary below p and shifted into place: a load whose address
// is not a multiple of 4 costs the cache nearly twice the accesses (measured).  Normal cached
// loads: the windows overlap.
//
// In two halves, so that a caller issues the loads of all its windows before it uses the
// first; the caller guarantees that the 20 bytes lie inside the array.  (With the load under a
// per-lane bounds test the compiler puts a full wait behind every one of them, and a wave's
// eight windows became eight trips to memory, one after the other; so the callers test a whole
// segment at once, wave-uniformly, and send the few segments at the very ends of the array
// through window_guarded in a loop of their own.)
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));

struct WindowLoad {
    u32x4 d;      // the four dwords from the dword boundary at or below p
    uint32_t d4;  // the fifth: the last value of a shifted window
};

// true when every window that starts in [first, last] can be read with window_issue
__device__ __forceinline__ bool windows_inside(uintptr_t first, uintptr_t last, uintptr_t vbeg, uintptr_t vend) {
    return (first & ~uintptr_t(3)) >= vbeg && last + 20 <= vend;
}

__device__ __forceinline__ WindowLoad window_issue(uintptr_t p) {
    const uintptr_t a = p & ~uintptr_t(3);
    WindowLoad L;
    L.d = *global_ptr<u32x4_a4>(a);
    L.d4 = *global_ptr<uint32_t>(a + 16);
    return L;
}

__device__ __forceinline__ u32x4 window_finish(const WindowLoad &L, uintptr_t p) {
    const uint32_t sh = static_cast<uint32_t>(p) & 3u;  // 0 or 2
    u32x4 w;
    w.x = __builtin_amdgcn_alignbyte(L.d.y, L.d.x, sh);
    w.y = __builtin_amdgcn_alignbyte(L.d.z, L.d.y, sh);
    w.z = __builtin_amdgcn_alignbyte(L.d.w, L.d.z, sh);
    w.w = __builtin_amdgcn_alignbyte(L.d4, L.d.w, sh);
    return w;
}

// The same window element by element, with bytes outside [vbeg, vend) read as 0.
__device__ __forceinline__ u32x4 window_guarded(uintptr_t p, uintptr_t vbeg, uintptr_t vend) {
    uint32_t d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uintptr_t q = p + 2 * j;
        uint32_t v = 0;
        if (q >= vbeg && q + 2 <= vend) v = *global_ptr<uint16_t>(q);
        d[j >> 1] |= v << (16 * (j & 1));
    }
    u32x4 w;
    w.x = d[0];
    w.y = d[1];
    w.z = d[2];
    w.w = d[3];
    return w;
}

}  // namespace endor_device

#endif  // ENDOR_DEVICE_H_
