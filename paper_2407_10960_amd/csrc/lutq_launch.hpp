// Host-side launch entry points, one pair per (bit width, dtype); each is defined by compiling
// lutq_kernels.hip with -DLUTQ_INST_BITS=<b> -DLUTQ_INST_DT=<F16|BF16>.
#pragma once

#include <hip/hip_runtime.h>

#include "lutq_matmul_kernel.hpp"

namespace lutq {

// Kernel instances that exist: waves per workgroup x tiles in flight.  (The per-tile scale path,
// used only when K/group is not a multiple of 8, exists for 4 waves and 2 tiles in flight.)
inline bool matmul_instance_exists(int nw, int stages, bool sch) {
    if (!sch) return nw == 4 && stages == 2;
    return (nw == 4 || nw == 8) && (stages == 2 || stages == 4);
}

#define LUTQ_DECLARE_LAUNCHERS(B, DT)                                                               \
    hipError_t launch_matmul_b##B##_##DT(int group, int mb, int r, int nw, int stages, bool sch,     \
                                         int xm, const MatmulParams& p, hipStream_t stream);         \
    hipError_t launch_dequant_b##B##_##DT(int group, const DequantParams& p, int grid, int lds_bytes, \
                                          hipStream_t stream);

LUTQ_DECLARE_LAUNCHERS(2, F16)
LUTQ_DECLARE_LAUNCHERS(3, F16)
LUTQ_DECLARE_LAUNCHERS(4, F16)
LUTQ_DECLARE_LAUNCHERS(2, BF16)
LUTQ_DECLARE_LAUNCHERS(3, BF16)
LUTQ_DECLARE_LAUNCHERS(4, BF16)

}  // namespace lutq
