// Instantiates the kernels for one (bit width, dtype) pair and dispatches the remaining template
// parameters (group size, M blocks, row blocks per wave) at run time.
#include "lutq_launch.hpp"

#ifndef LUTQ_INST_BITS
#error "compile with -DLUTQ_INST_BITS=2|3|4 -DLUTQ_INST_DT=F16|BF16"
#endif

#define LUTQ_CAT3(a, b, c) a##b##_##c
#define LUTQ_NAME(prefix, b, dt) LUTQ_CAT3(prefix, b, dt)

namespace lutq {

namespace {

template <int GROUP, int MB, int R>
hipError_t launch_one(const MatmulParams& p, int lds_bytes, hipStream_t stream) {
    hipLaunchKernelGGL((matmul_kernel<LUTQ_INST_BITS, GROUP, MB, R, LUTQ_INST_DT>), dim3(p.G), dim3(256), lds_bytes,
                       stream, p);
    return hipGetLastError();
}

template <int GROUP>
hipError_t launch_group(int mb, int r, const MatmulParams& p, int lds_bytes, hipStream_t stream) {
    if (mb == 1) {
        if (r == 1) return launch_one<GROUP, 1, 1>(p, lds_bytes, stream);
        if (r == 2) return launch_one<GROUP, 1, 2>(p, lds_bytes, stream);
        if (r == 4) return launch_one<GROUP, 1, 4>(p, lds_bytes, stream);
    } else if (mb == 2) {
        if (r == 1) return launch_one<GROUP, 2, 1>(p, lds_bytes, stream);
        if (r == 2) return launch_one<GROUP, 2, 2>(p, lds_bytes, stream);
        if (r == 4) return launch_one<GROUP, 2, 4>(p, lds_bytes, stream);
    }
    return hipErrorInvalidValue;
}

template <int GROUP>
hipError_t launch_dq(const DequantParams& p, int grid, int lds_bytes, hipStream_t stream) {
    hipLaunchKernelGGL((dequant_kernel<LUTQ_INST_BITS, GROUP, LUTQ_INST_DT>), dim3(grid), dim3(256), lds_bytes, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t LUTQ_NAME(launch_matmul_b, LUTQ_INST_BITS, LUTQ_INST_DT)(int group, int mb, int r, const MatmulParams& p,
                                                                    int lds_bytes, hipStream_t stream) {
    switch (group) {
        case 32: return launch_group<32>(mb, r, p, lds_bytes, stream);
        case 64: return launch_group<64>(mb, r, p, lds_bytes, stream);
        case 128: return launch_group<128>(mb, r, p, lds_bytes, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t LUTQ_NAME(launch_dequant_b, LUTQ_INST_BITS, LUTQ_INST_DT)(int group, const DequantParams& p, int grid,
                                                                     int lds_bytes, hipStream_t stream) {
    switch (group) {
        case 32: return launch_dq<32>(p, grid, lds_bytes, stream);
        case 64: return launch_dq<64>(p, grid, lds_bytes, stream);
        case 128: return launch_dq<128>(p, grid, lds_bytes, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace lutq
