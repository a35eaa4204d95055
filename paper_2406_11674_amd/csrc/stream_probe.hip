// Plain streaming kernels that measure what this MI355X's memory system delivers for the
// access mixes of the decompression path: write only, read only, copy, the 1.125 : 2
// read : write mix of decompression at half density (Section 4.1's sizes: 1/8 byte of bitmap
// and 1 byte of values read per 2 bytes written), and the same for any other ratio (other
// densities, 8-bit values).  They are a yardstick for the benchmark,
// not part of the decompression path, and live in a library of their own
// (libendor_probe.so) that only bench.py loads.
//
// Every kernel uses the shape that measured fastest for plain streaming on this part: one
// 16-byte unit per thread, 256 threads per workgroup, non-temporal accesses.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void probe_write(u32x4 *out, size_t units) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= units) return;
    u32x4 v;
    v.x = 1;
    v.y = 2;
    v.z = 3;
    v.w = uint32_t(i);
    __builtin_nontemporal_store(v, out + i);
}

// the loaded data feeds a store that never happens for real inputs, so the loads stay
__global__ __launch_bounds__(256) void probe_read(const u32x4 *in, size_t units, uint32_t *sink) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= units) return;
    const u32x4 v = __builtin_nontemporal_load(in + i);
    if ((v.x & v.y & v.z & v.w) == 0xdeadbeefu) *sink = v.x;
}

__global__ __launch_bounds__(256) void probe_copy(const u32x4 *in, u32x4 *out, size_t units) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= units) return;
    __builtin_nontemporal_store(__builtin_nontemporal_load(in + i), out + i);
}

// 9 units read for every 16 written: 1.125 bytes in per 2 bytes out
__global__ __launch_bounds__(256) void probe_mix(const u32x4 *in, u32x4 *out, size_t units) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= units) return;
    u32x4 v;
    v.x = v.y = v.z = v.w = uint32_t(i);
    if ((i & 15) < 9) v = __builtin_nontemporal_load(in + (i >> 4) * 9 + (i & 15));
    __builtin_nontemporal_store(v, out + i);
}

// k units read for every 256 written, for any k in 0..256: a workgroup writes its 256 units and
// its first k threads read the workgroup's contiguous run of the input (like a tile's value
// slice, it shares its first and last 128-byte line with the neighbours').  The stores do not
// wait for the loads, so the figure is what the memory system delivers for the mix, not what a
// dependent chain allows.
__global__ __launch_bounds__(256) void probe_mix_k(const u32x4 *in, u32x4 *out, size_t units, uint32_t k,
                                                   uint32_t *sink) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= units) return;
    u32x4 v;
    v.x = v.y = v.z = v.w = uint32_t(i);
    __builtin_nontemporal_store(v, out + i);
    if (threadIdx.x < k) {
        const u32x4 r = __builtin_nontemporal_load(in + size_t(blockIdx.x) * k + threadIdx.x);
        if ((r.x & r.y & r.z & r.w) == 0xdeadbeefu) *sink = r.x;
    }
}

}  // namespace

// kind: 0 write `bytes` to d_out; 1 read `bytes` from d_in; 2 copy `bytes` from d_in to d_out;
// 3 write `bytes` to d_out while reading bytes*9/16 from d_in.  bytes must be a multiple of
// 256 and below 2^40; d_in / d_out 16-byte aligned device buffers of at least `bytes` bytes;
// d_sink a device word.  Returns 0, or 1 on bad arguments, 2 on a launch error.
extern "C" int endor_probe_stream(int kind, const void *d_in, void *d_out, size_t bytes, void *d_sink, void *stream) {
    if (kind < 0 || kind > 3 || bytes == 0 || bytes % 256 != 0 || (bytes >> 40) != 0) return 1;
    if ((kind != 0 && !d_in) || (kind != 1 && !d_out) || (kind == 1 && !d_sink)) return 1;
    if ((reinterpret_cast<uintptr_t>(d_in) & 15) || (reinterpret_cast<uintptr_t>(d_out) & 15)) return 1;
    const size_t units = bytes / 16;
    const dim3 grid(static_cast<unsigned>((units + 255) / 256)), block(256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const u32x4 *in = static_cast<const u32x4 *>(d_in);
    u32x4 *out = static_cast<u32x4 *>(d_out);
    switch (kind) {
        case 0: hipLaunchKernelGGL(probe_write, grid, block, 0, s, out, units); break;
        case 1: hipLaunchKernelGGL(probe_read, grid, block, 0, s, in, units, static_cast<uint32_t *>(d_sink)); break;
        case 2: hipLaunchKernelGGL(probe_copy, grid, block, 0, s, in, out, units); break;
        default: hipLaunchKernelGGL(probe_mix, grid, block, 0, s, in, out, units); break;
    }
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// Writes `bytes` (a multiple of 4096) to d_out while reading bytes*reads_per_256/256 from d_in
// (reads_per_256 in 0..256).  Otherwise the argument rules of endor_probe_stream.
extern "C" int endor_probe_mix(int reads_per_256, const void *d_in, void *d_out, size_t bytes, void *d_sink,
                               void *stream) {
    if (reads_per_256 < 0 || reads_per_256 > 256 || bytes == 0 || bytes % 4096 != 0 || (bytes >> 40) != 0) return 1;
    if (!d_in || !d_out || !d_sink) return 1;
    if ((reinterpret_cast<uintptr_t>(d_in) & 15) || (reinterpret_cast<uintptr_t>(d_out) & 15)) return 1;
    const size_t units = bytes / 16;
    hipLaunchKernelGGL(probe_mix_k, dim3(static_cast<unsigned>(units / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const u32x4 *>(d_in), static_cast<u32x4 *>(d_out),
                       units, static_cast<uint32_t>(reads_per_256), static_cast<uint32_t *>(d_sink));
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
