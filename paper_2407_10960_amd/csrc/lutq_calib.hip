// Measurement helpers (not part of the method): a read-only streaming kernel and a plain copy kernel
// of known size.  The first gives the HBM read bandwidth a kernel of the same grid shape can reach;
// the second calibrates the profiler's byte counters against a known traffic volume.
#include <hip/hip_runtime.h>

#include "lutq_calib.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* sink) {
    const size_t stride = (size_t)gridDim.x * 256;
    u32x4 acc = u32x4{0u, 0u, 0u, 0u};
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 a = __builtin_nontemporal_load(src + i);
        const u32x4 b = __builtin_nontemporal_load(src + i + stride);
        const u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride);
        const u32x4 d = __builtin_nontemporal_load(src + i + 3 * stride);
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    const uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (r == 0x9e3779b9u) *sink = r;      // practically never true: keeps the loads alive
}

__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

extern "C" int lutq_calib_stream_read(const void* src, size_t bytes, int grid, void* sink4, void* stream) {
    if (!src || !sink4 || grid < 1 || (reinterpret_cast<uintptr_t>(src) & 15u)) return 1;
    hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(src), bytes / 16, static_cast<uint32_t*>(sink4));
    return hipGetLastError() == hipSuccess ? 0 : 9;
}

extern "C" int lutq_calib_copy(const void* src, void* dst, size_t bytes, int grid, void* stream) {
    if (!src || !dst || grid < 1 || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u)) return 1;
    hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : 9;
}
