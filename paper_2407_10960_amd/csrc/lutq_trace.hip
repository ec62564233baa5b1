// Measurement builds of the fused kernel: the same code with device timestamps at the phase boundaries
// (argument fetch, prefetch issued, table built, first tile, K loop, reduction, end), for the few
// instances the M <= 4 default plans of 4-bit weights use.  Launched only by lutq_calib_matmul_trace.
#include "lutq_launch.hpp"

namespace lutq {

namespace {

template <int GROUP, int R, typename DT>
hipError_t launch_traced(const MatmulParams& p, hipStream_t stream) {
    auto kernel = matmul_kernel<4, GROUP, 1, R, DT, 2, true, 4, true, 0, false, true>;
    const int lds_bytes = matmul_lds_bytes<4>(R, 1, p.NW, p.RS, true, false);
    if (lds_bytes > 64 * 1024) {
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (attr != hipSuccess) return attr;
    }
    hipLaunchKernelGGL(kernel, dim3(p.G), dim3(p.NW * 64), lds_bytes, stream, p);
    return hipGetLastError();
}

template <typename DT>
hipError_t launch_traced_dt(int group, int r, const MatmulParams& p, hipStream_t stream) {
    if (group == 64 && r == 1) return launch_traced<64, 1, DT>(p, stream);
    if (group == 64 && r == 2) return launch_traced<64, 2, DT>(p, stream);
    if (group == 128 && r == 1) return launch_traced<128, 1, DT>(p, stream);
    if (group == 128 && r == 2) return launch_traced<128, 2, DT>(p, stream);
    return hipErrorInvalidValue;
}

template <int GROUP, int R, typename DT>
hipError_t launch_decode_traced(const DecodeParams& p, int lds_bytes, hipStream_t stream) {
    auto kernel = decode_kernel<4, GROUP, R, DT, 2, true>;
    if (lds_bytes > 64 * 1024) {
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (attr != hipSuccess) return attr;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)p.G), dim3(p.NW * 64), lds_bytes, stream, p);
    return hipGetLastError();
}

template <typename DT>
hipError_t launch_decode_traced_dt(int group, int r, const DecodeParams& p, int lds_bytes, hipStream_t stream) {
    if (group == 64 && r == 1) return launch_decode_traced<64, 1, DT>(p, lds_bytes, stream);
    if (group == 64 && r == 2) return launch_decode_traced<64, 2, DT>(p, lds_bytes, stream);
    if (group == 128 && r == 1) return launch_decode_traced<128, 1, DT>(p, lds_bytes, stream);
    if (group == 128 && r == 2) return launch_decode_traced<128, 2, DT>(p, lds_bytes, stream);
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_decode_trace(bool bf16, int group, int r, const DecodeParams& p, int lds_bytes, hipStream_t stream) {
    return bf16 ? launch_decode_traced_dt<BF16>(group, r, p, lds_bytes, stream)
                : launch_decode_traced_dt<F16>(group, r, p, lds_bytes, stream);
}

hipError_t launch_matmul_trace(bool bf16, int group, int r, const MatmulParams& p, hipStream_t stream) {
    return bf16 ? launch_traced_dt<BF16>(group, r, p, stream) : launch_traced_dt<F16>(group, r, p, stream);
}

}  // namespace lutq
