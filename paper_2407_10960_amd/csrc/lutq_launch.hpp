// Host-side launch entry points, one pair per (bit width, dtype); each is defined by compiling
// lutq_kernels.hip with -DLUTQ_INST_BITS=<b> -DLUTQ_INST_DT=<F16|BF16>.
#pragma once

#include <hip/hip_runtime.h>

#include "lutq_matmul_kernel.hpp"

namespace lutq {

#define LUTQ_DECLARE_LAUNCHERS(B, DT)                                                                   \
    hipError_t launch_matmul_b##B##_##DT(int group, int mb, int r, int nw, bool sch, const MatmulParams& p,    \
                                         int lds_bytes, hipStream_t stream);                                            \
    hipError_t launch_dequant_b##B##_##DT(int group, const DequantParams& p, int grid, int lds_bytes,     \
                                          hipStream_t stream);

LUTQ_DECLARE_LAUNCHERS(2, F16)
LUTQ_DECLARE_LAUNCHERS(3, F16)
LUTQ_DECLARE_LAUNCHERS(4, F16)
LUTQ_DECLARE_LAUNCHERS(2, BF16)
LUTQ_DECLARE_LAUNCHERS(3, BF16)
LUTQ_DECLARE_LAUNCHERS(4, BF16)

}  // namespace lutq
