// Host-side launch entry points, one pair per (bit width, dtype); each is defined by compiling
// lutq_kernels.hip with -DLUTQ_INST_BITS=<b> -DLUTQ_INST_DT=<F16|BF16>.
#pragma once

#include <hip/hip_runtime.h>

#include "lutq_matmul_kernel.hpp"
#include "lutq_decode_kernel.hpp"
#include "lutq_rows_kernel.hpp"

namespace lutq {

// Kernel instances that exist.  `wide` instances run up to 16 waves per workgroup within 128
// registers and exist only where the register estimate fits; the others run up to 8 waves.  The
// per-tile scale path (K/group not a multiple of 8) exists for 2 tiles in flight, not wide.
// xsh: 0, or the number of activation pieces a wave stages (1 or 2) in a shared-activation instance
inline bool matmul_instance_exists(int bits, bool bf16, int r, int mb, int stages, bool sch, int xm, bool wide,
                                   int xsh = 0) {
    const bool wt = bf16 && bits != 2;                  // widened table: a larger lookup ring
    if (xsh && (xm != 16 || !sch)) return false;
    if (stages != 2 && stages != 4) return false;
    if (!sch) return stages == 2 && !wide;
    if (!wide) {                                        // up to 256 registers; beyond that the K loop would spill
        const int est = bits == 2 ? matmul_reg_estimate<2>(r, mb, stages, xm, wt, xsh)
                      : bits == 3 ? matmul_reg_estimate<3>(r, mb, stages, xm, wt, xsh) : matmul_reg_estimate<4>(r, mb, stages, xm, wt, xsh);
        return est <= 250;
    }
    return bits == 2 ? matmul_wide_fits<2>(r, mb, stages, xm, wt, xsh)
         : bits == 3 ? matmul_wide_fits<3>(r, mb, stages, xm, wt, xsh) : matmul_wide_fits<4>(r, mb, stages, xm, wt, xsh);
}

#define LUTQ_DECLARE_LAUNCHERS(B, DT)                                                               \
    hipError_t launch_matmul_b##B##_##DT(int group, int mb, int r, int stages, bool sch, int xm,     \
                                         bool wide, int xsh, const MatmulParams& p,                  \
                                         hipStream_t stream);                                        \
    hipError_t launch_matmul_rowlut_b##B##_##DT(int group, int mb, bool sch, int xm, const MatmulParams& p, \
                                                hipStream_t stream);                                 \
    hipError_t launch_dequant_b##B##_##DT(int group, const DequantParams& p, int grid, int lds_bytes, \
                                          hipStream_t stream);                                       \
    hipError_t launch_decode_b##B##_##DT(int group, int r, bool rowlut, const DecodeParams& p, int lds_bytes, \
                                         hipStream_t stream);                                        \
    hipError_t launch_rows_b##B##_##DT(int group, int mb, int amax, bool rowlut, const RowsParams& p, int lds_bytes, \
                                       hipStream_t stream);

// Measurement builds (phase timestamps, see TraceStamp) of the 4-bit instances that serve M <= 4 under the
// default plans: group 64 or 128, R = 1 or 2, two tiles in flight, chunked scales, 128-register build.
// Defined in lutq_trace.hip.
hipError_t launch_matmul_trace(bool bf16, int group, int r, const MatmulParams& p, hipStream_t stream);
// the same for the work-queue kernel (decode_kernel): 4-bit, group 64 or 128, R = 1 or 2
hipError_t launch_decode_trace(bool bf16, int group, int r, const DecodeParams& p, int lds_bytes, hipStream_t stream);

LUTQ_DECLARE_LAUNCHERS(2, F16)
LUTQ_DECLARE_LAUNCHERS(3, F16)
LUTQ_DECLARE_LAUNCHERS(4, F16)
LUTQ_DECLARE_LAUNCHERS(2, BF16)
LUTQ_DECLARE_LAUNCHERS(3, BF16)
LUTQ_DECLARE_LAUNCHERS(4, BF16)

}  // namespace lutq
