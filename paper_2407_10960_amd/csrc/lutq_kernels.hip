// Instantiates the kernels for one (bit width, dtype) pair and dispatches the remaining template
// parameters (group size, M blocks, row blocks per wave, tiles in flight, scale path, activation
// packing, register budget) at run time.
#include "lutq_launch.hpp"

#ifndef LUTQ_INST_BITS
#error "compile with -DLUTQ_INST_BITS=2|3|4 -DLUTQ_INST_DT=F16|BF16"
#endif

#define LUTQ_CAT3(a, b, c) a##b##_##c
#define LUTQ_NAME(prefix, b, dt) LUTQ_CAT3(prefix, b, dt)

namespace lutq {

namespace {

template <int GROUP, int MB, int R, int P, bool SCH, int XM, bool WIDE, int XSH>
hipError_t launch_one(const MatmulParams& p, hipStream_t stream) {
    constexpr bool wide_table = Tab<LUTQ_INST_BITS, LUTQ_INST_DT>::WIDE;
    if constexpr (WIDE && !matmul_wide_fits<LUTQ_INST_BITS>(R, MB, P, XM, wide_table, XSH)) {
        return hipErrorInvalidValue;         // would not fit 128 registers: not instantiated
    } else {
        auto kernel = matmul_kernel<LUTQ_INST_BITS, GROUP, MB, R, LUTQ_INST_DT, P, SCH, XM, WIDE, XSH>;
        const int lds_bytes = matmul_lds_bytes<LUTQ_INST_BITS>(R, MB, p.NW, p.RS, SCH, XSH != 0);
        if (lds_bytes > 64 * 1024) {
            // more than 64 KiB of dynamic LDS has to be enabled once per kernel
            static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (attr != hipSuccess) return attr;
        }
        hipLaunchKernelGGL(kernel, dim3(p.G), dim3(p.NW * 64), lds_bytes, stream, p);
        return hipGetLastError();
    }
}

// xsh: 0 = every wave fetches its own activations; 1 or 2 = activations shared through LDS, that many
// pieces of a tile staged per wave
template <int GROUP, int MB, int R, int P, int XSH>
hipError_t launch_shared(bool wide, const MatmulParams& p, hipStream_t stream) {
    return wide ? launch_one<GROUP, MB, R, P, true, 16, true, XSH>(p, stream)
                : launch_one<GROUP, MB, R, P, true, 16, false, XSH>(p, stream);
}

template <int GROUP, int MB, int R, int XM>
hipError_t launch_r(int stages, bool sch, bool wide, int xsh, const MatmulParams& p, hipStream_t stream) {
    if constexpr (XM == 16) {
        // activations shared through LDS: chunked scales
        if (xsh) {
            if (!sch) return hipErrorInvalidValue;
            if (stages == 2 && xsh == 1) return launch_shared<GROUP, MB, R, 2, 1>(wide, p, stream);
            if (stages == 2 && xsh == 2) return launch_shared<GROUP, MB, R, 2, 2>(wide, p, stream);
            if (stages == 4 && xsh == 1) return launch_shared<GROUP, MB, R, 4, 1>(wide, p, stream);
            if (stages == 4 && xsh == 2) return launch_shared<GROUP, MB, R, 4, 2>(wide, p, stream);
            return hipErrorInvalidValue;
        }
    } else if (xsh) {
        return hipErrorInvalidValue;
    }
    if (!sch) return (!wide && stages == 2) ? launch_one<GROUP, MB, R, 2, false, XM, false, 0>(p, stream) : hipErrorInvalidValue;
    if (wide) {
        if (stages == 2) return launch_one<GROUP, MB, R, 2, true, XM, true, 0>(p, stream);
        if (stages == 4) return launch_one<GROUP, MB, R, 4, true, XM, true, 0>(p, stream);
    } else {
        if (stages == 2) return launch_one<GROUP, MB, R, 2, true, XM, false, 0>(p, stream);
        if (stages == 4) return launch_one<GROUP, MB, R, 4, true, XM, false, 0>(p, stream);
    }
    return hipErrorInvalidValue;
}

template <int GROUP>
hipError_t launch_group(int mb, int r, int stages, bool sch, int xm, bool wide, int xsh, const MatmulParams& p, hipStream_t stream) {
    if (mb == 1 && xm == 4) {
        if (r == 1) return launch_r<GROUP, 1, 1, 4>(stages, sch, wide, xsh, p, stream);
        if (r == 2) return launch_r<GROUP, 1, 2, 4>(stages, sch, wide, xsh, p, stream);
        if (r == 4) return launch_r<GROUP, 1, 4, 4>(stages, sch, wide, xsh, p, stream);
    } else if (mb == 1 && xm == 8) {
        if (r == 1) return launch_r<GROUP, 1, 1, 8>(stages, sch, wide, xsh, p, stream);
        if (r == 2) return launch_r<GROUP, 1, 2, 8>(stages, sch, wide, xsh, p, stream);
        if (r == 4) return launch_r<GROUP, 1, 4, 8>(stages, sch, wide, xsh, p, stream);
    } else if (mb == 1 && xm == 16) {
        if (r == 1) return launch_r<GROUP, 1, 1, 16>(stages, sch, wide, xsh, p, stream);
        if (r == 2) return launch_r<GROUP, 1, 2, 16>(stages, sch, wide, xsh, p, stream);
        if (r == 4) return launch_r<GROUP, 1, 4, 16>(stages, sch, wide, xsh, p, stream);
    } else if (mb == 2 && xm == 16) {
        if (r == 1) return launch_r<GROUP, 2, 1, 16>(stages, sch, wide, xsh, p, stream);
        if (r == 2) return launch_r<GROUP, 2, 2, 16>(stages, sch, wide, xsh, p, stream);
        if (r == 4) return launch_r<GROUP, 2, 4, 16>(stages, sch, wide, xsh, p, stream);
    }
    return hipErrorInvalidValue;
}

// One table per output row: R = 1, one team, two tiles in flight; the 128-register build where it fits.
template <int GROUP, int MB, int XM, bool SCH>
hipError_t launch_rowlut_one(const MatmulParams& p, hipStream_t stream) {
    constexpr bool wide_table = Tab<LUTQ_INST_BITS, LUTQ_INST_DT>::WIDE;
    constexpr bool WIDE = SCH && matmul_wide_fits<LUTQ_INST_BITS>(1, MB, 2, XM, wide_table, 0);
    auto kernel = matmul_kernel<LUTQ_INST_BITS, GROUP, MB, 1, LUTQ_INST_DT, 2, SCH, XM, WIDE, 0, true>;
    const int lds_bytes = matmul_lds_bytes<LUTQ_INST_BITS>(1, MB, p.NW, p.RS, SCH, false);
    if (p.RS != 1 || p.NW > (WIDE ? 16 : 8)) return hipErrorInvalidValue;
    if (lds_bytes > 64 * 1024) {
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (attr != hipSuccess) return attr;
    }
    hipLaunchKernelGGL(kernel, dim3(p.G), dim3(p.NW * 64), lds_bytes, stream, p);
    return hipGetLastError();
}

template <int GROUP>
hipError_t launch_rowlut(int mb, int xm, bool sch, const MatmulParams& p, hipStream_t stream) {
    if (mb == 1 && xm == 4) return sch ? launch_rowlut_one<GROUP, 1, 4, true>(p, stream) : launch_rowlut_one<GROUP, 1, 4, false>(p, stream);
    if (mb == 1 && xm == 8) return sch ? launch_rowlut_one<GROUP, 1, 8, true>(p, stream) : launch_rowlut_one<GROUP, 1, 8, false>(p, stream);
    if (mb == 1 && xm == 16) return sch ? launch_rowlut_one<GROUP, 1, 16, true>(p, stream) : launch_rowlut_one<GROUP, 1, 16, false>(p, stream);
    if (mb == 2 && xm == 16) return sch ? launch_rowlut_one<GROUP, 2, 16, true>(p, stream) : launch_rowlut_one<GROUP, 2, 16, false>(p, stream);
    return hipErrorInvalidValue;
}

// Work-queue kernel for M <= 4: two tiles in flight, R = 1 or 2; RLUT: one table per output row (R = 1).
template <int GROUP, int R, bool RLUT = false>
hipError_t launch_decode_one(const DecodeParams& p, int lds_bytes, hipStream_t stream) {
    if constexpr (!decode_instance_exists(LUTQ_INST_BITS, Tab<LUTQ_INST_BITS, LUTQ_INST_DT>::WIDE, R)) {
        return hipErrorInvalidValue;
    } else {
    auto kernel = decode_kernel<LUTQ_INST_BITS, GROUP, R, LUTQ_INST_DT, 2, false, RLUT>;
    if (lds_bytes > 64 * 1024) {
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (attr != hipSuccess) return attr;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)p.G), dim3(p.NW * 64), lds_bytes, stream, p);
    return hipGetLastError();
    }
}

template <int GROUP>
hipError_t launch_decode_group(int r, bool rowlut, const DecodeParams& p, int lds_bytes, hipStream_t stream) {
    if (rowlut) return r == 1 ? launch_decode_one<GROUP, 1, true>(p, lds_bytes, stream) : hipErrorInvalidValue;
    if (r == 1) return launch_decode_one<GROUP, 1>(p, lds_bytes, stream);
    if (r == 2) return launch_decode_one<GROUP, 2>(p, lds_bytes, stream);
    return hipErrorInvalidValue;
}

// Row-streaming kernel for 5..64 activation rows: MB blocks of sixteen rows, AMAX = 4 or 8 row blocks side by side.
template <int GROUP, int MB, int AMAX, bool RLUT = false>
hipError_t launch_rows_one(const RowsParams& p, int lds_bytes, hipStream_t stream) {
    constexpr int max_waves = rows_max_waves(LUTQ_INST_BITS, MB, AMAX, Tab<LUTQ_INST_BITS, LUTQ_INST_DT>::WIDE);
    if constexpr (max_waves == 0) {
        return hipErrorInvalidValue;
    } else {
        if (p.NW > max_waves) return hipErrorInvalidValue;
        auto kernel = rows_kernel<LUTQ_INST_BITS, GROUP, MB, LUTQ_INST_DT, AMAX, RLUT>;
        if (lds_bytes > 64 * 1024) {
            static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (attr != hipSuccess) return attr;
        }
        hipLaunchKernelGGL(kernel, dim3((unsigned)p.G), dim3(p.NW * 64), lds_bytes, stream, p);
        return hipGetLastError();
    }
}

template <int GROUP>
hipError_t launch_rows_group(int mb, int amax, bool rowlut, const RowsParams& p, int lds_bytes, hipStream_t stream) {
    if (rowlut) {                    // one table per output row: four row blocks side by side
        if (mb == 1 && amax == 4) return launch_rows_one<GROUP, 1, 4, true>(p, lds_bytes, stream);
        if (mb == 2 && amax == 4) return launch_rows_one<GROUP, 2, 4, true>(p, lds_bytes, stream);
        return hipErrorInvalidValue;
    }
    if (mb == 1 && amax == 4) return launch_rows_one<GROUP, 1, 4>(p, lds_bytes, stream);
    if (mb == 1 && amax == 8) return launch_rows_one<GROUP, 1, 8>(p, lds_bytes, stream);
    if (mb == 2 && amax == 4) return launch_rows_one<GROUP, 2, 4>(p, lds_bytes, stream);
    if (mb == 2 && amax == 8) return launch_rows_one<GROUP, 2, 8>(p, lds_bytes, stream);
    if (mb == 3 && amax == 4) return launch_rows_one<GROUP, 3, 4>(p, lds_bytes, stream);   // 33..64 rows (4 bits)
    if (mb == 4 && amax == 4) return launch_rows_one<GROUP, 4, 4>(p, lds_bytes, stream);
    return hipErrorInvalidValue;
}

template <int GROUP>
hipError_t launch_dq(const DequantParams& p, int grid, int lds_bytes, hipStream_t stream) {
    hipLaunchKernelGGL((dequant_kernel<LUTQ_INST_BITS, GROUP, LUTQ_INST_DT>), dim3(grid), dim3(256), lds_bytes, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t LUTQ_NAME(launch_matmul_b, LUTQ_INST_BITS, LUTQ_INST_DT)(int group, int mb, int r, int stages, bool sch,
                                                                    int xm, bool wide, int xsh,
                                                                    const MatmulParams& p, hipStream_t stream) {
    switch (group) {
        case 32: return launch_group<32>(mb, r, stages, sch, xm, wide, xsh, p, stream);
        case 64: return launch_group<64>(mb, r, stages, sch, xm, wide, xsh, p, stream);
        case 128: return launch_group<128>(mb, r, stages, sch, xm, wide, xsh, p, stream);
        case 256: return launch_group<256>(mb, r, stages, sch, xm, wide, xsh, p, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t LUTQ_NAME(launch_matmul_rowlut_b, LUTQ_INST_BITS, LUTQ_INST_DT)(int group, int mb, bool sch, int xm,
                                                                           const MatmulParams& p, hipStream_t stream) {
    switch (group) {
        case 32: return launch_rowlut<32>(mb, xm, sch, p, stream);
        case 64: return launch_rowlut<64>(mb, xm, sch, p, stream);
        case 128: return launch_rowlut<128>(mb, xm, sch, p, stream);
        case 256: return launch_rowlut<256>(mb, xm, sch, p, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t LUTQ_NAME(launch_decode_b, LUTQ_INST_BITS, LUTQ_INST_DT)(int group, int r, bool rowlut, const DecodeParams& p, int lds_bytes,
                                                                    hipStream_t stream) {
    switch (group) {
        case 32: return launch_decode_group<32>(r, rowlut, p, lds_bytes, stream);
        case 64: return launch_decode_group<64>(r, rowlut, p, lds_bytes, stream);
        case 128: return launch_decode_group<128>(r, rowlut, p, lds_bytes, stream);
        case 256: return launch_decode_group<256>(r, rowlut, p, lds_bytes, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t LUTQ_NAME(launch_rows_b, LUTQ_INST_BITS, LUTQ_INST_DT)(int group, int mb, int amax, bool rowlut, const RowsParams& p, int lds_bytes,
                                                                  hipStream_t stream) {
    switch (group) {
        case 32: return launch_rows_group<32>(mb, amax, rowlut, p, lds_bytes, stream);
        case 64: return launch_rows_group<64>(mb, amax, rowlut, p, lds_bytes, stream);
        case 128: return launch_rows_group<128>(mb, amax, rowlut, p, lds_bytes, stream);
        case 256: return launch_rows_group<256>(mb, amax, rowlut, p, lds_bytes, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t LUTQ_NAME(launch_dequant_b, LUTQ_INST_BITS, LUTQ_INST_DT)(int group, const DequantParams& p, int grid,
                                                                     int lds_bytes, hipStream_t stream) {
    switch (group) {
        case 32: return launch_dq<32>(p, grid, lds_bytes, stream);
        case 64: return launch_dq<64>(p, grid, lds_bytes, stream);
        case 128: return launch_dq<128>(p, grid, lds_bytes, stream);
        case 256: return launch_dq<256>(p, grid, lds_bytes, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace lutq
