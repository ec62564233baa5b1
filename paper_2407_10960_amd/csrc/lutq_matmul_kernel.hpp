// The fused kernel: stream packed weights HBM -> registers, dequantise through the LDS table,
// scale, multiply on the matrix cores, reduce partial sums across workgroups.
//
// Follows Algorithm 1 / Algorithm 2 of the paper in what is computed; the data path is
// re-designed for gfx950:
//   * weights never pass through LDS: the offline layout makes a wavefront's 128-bit global loads
//     land directly in A-operand order of v_mfma_f32_16x16x32 (weights on the A side, Y^T = W^ X^T);
//   * the only LDS resident is the vectorised table (Section 3.2), one private copy per bank column;
//   * M < 16 (or < 32) is padded with zero B-operand lanes in registers (the paper pads in shared
//     memory, "Limitations"), which costs no memory traffic;
//   * work is split Stream-K style (Section 3.3): the (row group x K tile) iteration space is cut
//     into `grid` equal contiguous ranges, so a workgroup's range may start and end in the middle of
//     an output tile.  Partial sums go to a global scratch slot per (workgroup, end); an arrival
//     counter per output tile elects the last contributor, which adds the slots in a fixed order
//     (bit-reproducible results), writes Y and resets the counter.  Nobody ever waits on another
//     workgroup, so the kernel cannot deadlock whatever the number of resident workgroups.
#pragma once

#include "lutq_device.hpp"

namespace lutq {

struct MatmulParams {
    const uint16_t* X;        // [M, K]
    const uint8_t* packed;
    const uint16_t* scales;   // [N, SG]
    const uint16_t* lut;
    uint16_t* Y;              // [M, N]
    uint32_t* counters;       // [NRG], zero on entry, zero on exit
    float* slots;             // [G][2][SLOT_FLOATS]
    int M, N, K;
    int KT;                   // K tiles per row block
    int NRG;                  // row groups (N / (16 R))
    int G;                    // workgroups
    int log2c;                // log2 of table copies
    int SG;                   // scales per row (K / group)
};

// Largest partial-sum slot: R = 4 row blocks x 2 M-halves x 4 registers x 64 lanes.
constexpr int kSlotFloats = 4 * 2 * 4 * 64;

// Workgroup that owns iteration t when T iterations are cut into G ranges [floor(gT/G), floor((g+1)T/G)).
__device__ __forceinline__ int owner_of(int64_t t, int64_t T, int G) {
    return (int)(((t + 1) * G - 1) / T);
}

template <int BITS, int GROUP, int MB, int R, typename DT>
__global__ __launch_bounds__(256) void matmul_kernel(const MatmulParams p) {
    using Gm = Geo<BITS>;
    constexpr int TK = Gm::TK, STEPS = Gm::STEPS, TILE_BYTES = Gm::TILE_BYTES;
    constexpr int NS = TK / GROUP;           // scales per tile per row
    constexpr int SPG = GROUP / 32;          // steps per group
    constexpr int NREG = R * MB * 4;         // accumulator registers per lane
    constexpr int P = 2;                     // tiles in flight per wave

    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15;                // row inside a 16-row block (A side) / activation row (B side)
    const int lo = lane >> 4;                // K octet

    char* lut = smem;
    float* red = reinterpret_cast<float*>(smem + lut_lds_bytes<BITS>(p.log2c));   // [3][NREG][64]

    build_lut<BITS>(lut, p.lut, p.log2c, tid);
    const LutAddr la = make_lut_addr<BITS>(lut, p.log2c, lane);
    __syncthreads();

    bool valid[MB];
    const uint16_t* xlane[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = li + 16 * mb;
        valid[mb] = m < p.M;
        xlane[mb] = p.X + (size_t)(valid[mb] ? m : 0) * p.K + 8 * lo;
    }

    const int64_t T = (int64_t)p.NRG * p.KT;
    int64_t t0 = (int64_t)blockIdx.x * T / p.G;
    const int64_t t1 = (int64_t)(blockIdx.x + 1) * T / p.G;
    const int64_t tbeg = t0;

    struct Stage {
        WFrag<BITS> w[R];
        ScaleWords<NS> s[R];
        u32x4 x[STEPS][MB];
    };

    while (t0 < t1) {
        const int rg = (int)(t0 / p.KT);
        const int ka = (int)(t0 - (int64_t)rg * p.KT);
        const int rem = (int)((t1 - t0 < (int64_t)(p.KT - ka)) ? (t1 - t0) : (int64_t)(p.KT - ka));
        const int kb = ka + rem;
        const int wa = ka + (wave * rem) / 4;
        const int wb = ka + ((wave + 1) * rem) / 4;

        f32x4 acc[R][MB];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) acc[r][mb] = f32x4{0.f, 0.f, 0.f, 0.f};

        const uint8_t* wrow = p.packed + (size_t)rg * R * p.KT * TILE_BYTES;           // wave-uniform
        const uint16_t* srow = p.scales + ((size_t)rg * R * 16 + li) * p.SG;           // + r*16*SG per block

        auto load_stage = [&](Stage& st, int kt) {
#pragma unroll
            for (int r = 0; r < R; ++r)
                load_wfrag<BITS>(st.w[r], wrow + ((size_t)r * p.KT + kt) * TILE_BYTES, lane);
#pragma unroll
            for (int r = 0; r < R; ++r)
                load_scales<NS>(st.s[r], srow + (size_t)r * 16 * p.SG + (size_t)kt * NS);
#pragma unroll
            for (int s = 0; s < STEPS; ++s)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    u32x4 v = u32x4{0u, 0u, 0u, 0u};
                    if (valid[mb]) v = *reinterpret_cast<const u32x4*>(xlane[mb] + (size_t)kt * TK + 32 * s);
                    st.x[s][mb] = v;
                }
        };
        auto compute_stage = [&](const Stage& st) {
            // table reads of step s+1 are issued before step s is scaled and multiplied
            u32x4 raw[2][R];
#pragma unroll
            for (int r = 0; r < R; ++r) raw[0][r] = lookup_step<BITS>(st.w[r], 0, la);
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                if (s + 1 < STEPS) {
#pragma unroll
                    for (int r = 0; r < R; ++r) raw[(s + 1) & 1][r] = lookup_step<BITS>(st.w[r], s + 1, la);
                }
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const ScaleReg<DT> sc = make_scale<DT>(scale_bits<NS>(st.s[r], s / SPG));
                    const u32x4 a = scale4<DT>(raw[s & 1][r], sc);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) acc[r][mb] = mfma16x16x32<DT>(a, st.x[s][mb], acc[r][mb]);
                }
            }
        };

        Stage st[P];
#pragma unroll
        for (int q = 0; q < P; ++q)
            if (wa + q < wb) load_stage(st[q], wa + q);
        for (int kt = wa; kt < wb; kt += P) {
#pragma unroll
            for (int q = 0; q < P; ++q) {
                if (kt + q < wb) {
                    compute_stage(st[q]);
                    if (kt + q + P < wb) load_stage(st[q], kt + q + P);
                }
            }
        }

        // ---- reduce the four waves of the workgroup through LDS ----
        if (wave != 0) {
            float* dst = red + (size_t)(wave - 1) * NREG * 64 + lane;
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) dst[((r * MB + mb) * 4 + i) * 64] = acc[r][mb][i];
        }
        __syncthreads();
        if (wave == 0) {
            for (int w = 0; w < 3; ++w) {
                const float* src = red + (size_t)w * NREG * 64 + lane;
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int i = 0; i < 4; ++i) acc[r][mb][i] += src[((r * MB + mb) * 4 + i) * 64];
            }
        }
        __syncthreads();

        // ---- emit: whole output tile -> Y; otherwise the Stream-K fix-up ----
        if (wave == 0) {
            bool write_y = (ka == 0 && kb == p.KT);
            if (!write_y) {
                const int64_t tile0 = (int64_t)rg * p.KT;
                const int g_first = owner_of(tile0, T, p.G);
                const int g_last = owner_of(tile0 + p.KT - 1, T, p.G);
                const int which = (t0 == tbeg) ? 0 : 1;
                float* slot = p.slots + ((size_t)blockIdx.x * 2 + which) * kSlotFloats + lane;
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        if (valid[mb])
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                __hip_atomic_store(slot + ((r * MB + mb) * 4 + i) * 64, acc[r][mb][i],
                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __threadfence();       // partial sums visible device-wide before the arrival is counted
                uint32_t old = 0;
                if (lane == 0)
                    old = __hip_atomic_fetch_add(p.counters + rg, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
                old = __builtin_amdgcn_readfirstlane(old);
                if (old == (uint32_t)(g_last - g_first)) {
                    __threadfence();
                    // last contributor: add every slot in workgroup order (own one included)
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb) acc[r][mb] = f32x4{0.f, 0.f, 0.f, 0.f};
                    for (int g = g_first; g <= g_last; ++g) {
                        const int64_t gbeg = (int64_t)g * T / p.G;
                        const int gw = (gbeg / p.KT == rg) ? 0 : 1;     // slot 0 iff rg is g's first row group
                        const float* src = p.slots + ((size_t)g * 2 + gw) * kSlotFloats + lane;
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int mb = 0; mb < MB; ++mb)
                                if (valid[mb])
#pragma unroll
                                    for (int i = 0; i < 4; ++i)
                                        acc[r][mb][i] += __hip_atomic_load(src + ((r * MB + mb) * 4 + i) * 64,
                                                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    if (lane == 0)
                        __hip_atomic_store(p.counters + rg, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    write_y = true;
                }
            }
            if (write_y) {
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        if (valid[mb]) {
                            const int m = li + 16 * mb;
                            const int n = (rg * R + r) * 16 + 4 * lo;
                            *reinterpret_cast<u32x2*>(p.Y + (size_t)m * p.N + n) = pack4<DT>(acc[r][mb]);
                        }
            }
        }
        t0 += rem;
    }
}

// ---------------------------------------------------------------------------------------------
// Dequantise to memory (the separate-kernel baseline of Section 3): one wave per tile, same lookup
// and scale routine as the fused kernel.
// ---------------------------------------------------------------------------------------------
struct DequantParams {
    const uint8_t* packed;
    const uint16_t* scales;
    const uint16_t* lut;
    uint16_t* W;      // [N, K]
    int N, K, KT, SG;
    int64_t tiles;    // (N/16) * KT
    int log2c;
};

template <int BITS, int GROUP, typename DT>
__global__ __launch_bounds__(256) void dequant_kernel(const DequantParams p) {
    using Gm = Geo<BITS>;
    constexpr int TK = Gm::TK, STEPS = Gm::STEPS, TILE_BYTES = Gm::TILE_BYTES;
    constexpr int NS = TK / GROUP, SPG = GROUP / 32;
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    build_lut<BITS>(smem, p.lut, p.log2c, tid);
    const LutAddr la = make_lut_addr<BITS>(smem, p.log2c, lane);
    __syncthreads();
    const int li = lane & 15, lo = lane >> 4;
    for (int64_t t = (int64_t)blockIdx.x * 4 + wave; t < p.tiles; t += (int64_t)gridDim.x * 4) {
        const int64_t rb = t / p.KT;
        const int kt = (int)(t - rb * p.KT);
        WFrag<BITS> f;
        load_wfrag<BITS>(f, p.packed + (size_t)t * TILE_BYTES, lane);
        ScaleWords<NS> sw;
        load_scales<NS>(sw, p.scales + ((size_t)rb * 16 + li) * p.SG + (size_t)kt * NS);
        uint16_t* out = p.W + ((size_t)rb * 16 + li) * p.K + (size_t)kt * TK + 8 * lo;
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const ScaleReg<DT> sc = make_scale<DT>(scale_bits<NS>(sw, s / SPG));
            const u32x4 a = scale4<DT>(lookup_step<BITS>(f, s, la), sc);
            *reinterpret_cast<u32x4*>(out + 32 * s) = a;
        }
    }
}

}  // namespace lutq
