// GPU quantiser: dense weights -> table indices + group scales, written directly in the packed
// layout of lutq_pack.cpp (Section 3, first equation: Q = argmin_c |W/s - T[c]|; Section 4.1 "LUT
// quantization method" / Section 4.2: one absmax scale per group, stored in the 16-bit type; Section
// 3.1: the offline reordering, here fused into the same pass).
//
// Every decision is taken in fp64 on exactly representable inputs, so the result is a function of
// the inputs alone: the scale is the group's absmax rounded once (to nearest even) to the 16-bit
// type; u = W / scale is one IEEE fp64 division; the index is the first c that minimises the fp64
// value |u - T[c]|; a group whose scale is zero takes u = 0.
//
// The minimum is found by scanning all 2^b entries, except for a strictly increasing fp16 table of 8
// or 16 entries (the NormalFloat tables and sorted learned tables are; with 4 entries the scan is the
// faster of the two): there a binary search over a copy of the table in LDS brackets u between two neighbours and only their two distances are compared.  This gives
// the same index as the scan: |u| < 2 and fp16 magnitudes are at most 65504, so a distance
// is below 2^17 and its fp64 rounding error below 2^-36, while two different fp16 values are at least
// 2^-24 apart -- rounding keeps the distances to different entries in their exact order, the nearest
// entry is one of the two neighbours, and a tie between them goes to the lower one, which is the
// lower index.  bf16 values can be closer together than a rounding error, so bf16 tables are scanned.
//
// Work unit: 16 rows x UC columns, UC = max(K tile, group), one wavefront per unit.  Lane l = 16 o + i
// holds, for every 32-column step t of the unit, the 8 weights W[16 rb + i][col0 + 32 t + 8 o + j] --
// exactly the 8 indices whose packed bits this lane owns -- so the packed tile is written with one
// 128-bit store per lane (plus one 64-bit store for the 3-bit high slice) and needs no exchange; only
// the group maximum crosses lanes (the four lanes i, 16 + i, 32 + i, 48 + i share a row).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "lutq.h"
#include "lutq_layout.hpp"

namespace lutq {

struct QuantParams {
    const void* W;            // [N, K] fp32 or 16-bit
    const uint16_t* lut;      // 2^bits entries
    uint16_t* scales;         // [N, K / group]
    uint8_t* packed;
    int N, K, KT, SG, SB;     // KT = K / TK, SG = K / group, SB = row blocks per super-block
    int upr;                  // units per row block = K / UC
    long long units;
    int bf16;                 // 16-bit type of lut, scales (and of W unless fp32)
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float widen16(uint32_t h, bool bf16) {
    if (bf16) return __builtin_bit_cast(float, h << 16);
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}

// fp32 (finite, >= 0) -> 16-bit pattern, round to nearest even
__device__ __forceinline__ uint32_t round16(float v, bool bf16) {
    if (bf16) {
        const uint32_t b = __builtin_bit_cast(uint32_t, v);
        return (b + 0x7fffu + ((b >> 16) & 1u)) >> 16;
    }
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)v);
}

template <int BITS, int GROUP, bool WF32>
__global__ __launch_bounds__(256) void quantize_kernel(const QuantParams p) {
    constexpr int TK = BITS == 4 ? 128 : 256;
    constexpr int TILE_BYTES = BITS == 3 ? 1536 : 1024;
    constexpr int UC = GROUP > TK ? GROUP : TK;       // columns of one unit
    constexpr int NSTEP = UC / 32;                    // 32-column steps of one unit
    constexpr int STEPS = TK / 32;                    // steps of one tile
    constexpr int SPG = GROUP / 32;                   // steps of one group
    constexpr int NG = UC / GROUP;                    // groups of one unit (per row)
    constexpr int E = 1 << BITS;
    const bool bf16 = p.bf16 != 0;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, o = lane >> 4;

    double T[E];
#pragma unroll
    for (int c = 0; c < E; ++c) T[c] = (double)widen16(p.lut[c], bf16);
    __shared__ double Ts[E];
    bool sorted = !bf16 && BITS >= 3;
#pragma unroll
    for (int c = 0; c + 1 < E; ++c) sorted = sorted && T[c] < T[c + 1];
    if (threadIdx.x < E) {
        double v = T[0];
#pragma unroll
        for (int c = 1; c < E; ++c) v = (int)threadIdx.x == c ? T[c] : v;
        Ts[threadIdx.x] = v;
    }
    __syncthreads();

    for (long long unit = (long long)blockIdx.x * 4 + wave; unit < p.units; unit += (long long)gridDim.x * 4) {
        const int rb = (int)(unit / p.upr), uc = (int)(unit % p.upr);
        const long long row = 16ll * rb + i;
        const int col0 = uc * UC;
        float w[NSTEP][8];
#pragma unroll
        for (int t = 0; t < NSTEP; ++t) {
            const long long e = row * p.K + col0 + 32 * t + 8 * o;
            if constexpr (WF32) {
                const float4* src = reinterpret_cast<const float4*>(static_cast<const float*>(p.W) + e);
                const float4 a = src[0], b = src[1];
                w[t][0] = a.x; w[t][1] = a.y; w[t][2] = a.z; w[t][3] = a.w;
                w[t][4] = b.x; w[t][5] = b.y; w[t][6] = b.z; w[t][7] = b.w;
            } else {
                const u32x4 v = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.W) + e);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    w[t][2 * j] = widen16(v[j] & 0xffffu, bf16);
                    w[t][2 * j + 1] = widen16(v[j] >> 16, bf16);
                }
            }
        }
        // group maxima of |w| on the bit patterns (non-negative floats order like unsigned integers)
        uint32_t sbits[NG];
        double s[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            uint32_t m = 0;
#pragma unroll
            for (int t = g * SPG; t < (g + 1) * SPG; ++t)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t a = __builtin_bit_cast(uint32_t, w[t][j]) & 0x7fffffffu;
                    m = a > m ? a : m;
                }
            const uint32_t m1 = (uint32_t)__shfl_xor((int)m, 16);
            m = m1 > m ? m1 : m;
            const uint32_t m2 = (uint32_t)__shfl_xor((int)m, 32);
            m = m2 > m ? m2 : m;
            sbits[g] = round16(__builtin_bit_cast(float, m), bf16);
            s[g] = (double)widen16(sbits[g], bf16);
        }
        if (o == 0) {
            uint16_t* dst = p.scales + row * p.SG + (long long)uc * NG;
#pragma unroll
            for (int g = 0; g < NG; ++g) dst[g] = (uint16_t)sbits[g];
        }
        // indices of this lane, step by step, packed as they are found
        uint32_t idx[NSTEP];                          // 8 indices of step t, 4 bits apart
#pragma unroll
        for (int t = 0; t < NSTEP; ++t) {
            const double sg = s[t / SPG];
            uint32_t word = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const double u = sg == 0.0 ? 0.0 : (double)w[t][j] / sg;
                uint32_t arg = 0;
                if (sorted) {                               // (uniform over the launch)
                    int lower = 0;                          // entries [0, lower) are <= u
#pragma unroll
                    for (int step = E / 2; step >= 1; step >>= 1)
                        if (Ts[lower + step - 1] <= u) lower += step;
                    if (Ts[lower] <= u) lower += 1;
                    const int lo = lower > 0 ? lower - 1 : 0, hi = lower < E ? lower : E - 1;
                    arg = __builtin_fabs(u - Ts[hi]) < __builtin_fabs(u - Ts[lo]) ? (uint32_t)hi : (uint32_t)lo;
                } else {
                    double best = __builtin_fabs(u - T[0]);
#pragma unroll
                    for (int c = 1; c < E; ++c) {
                        const double d = __builtin_fabs(u - T[c]);
                        const bool less = d < best;
                        best = less ? d : best;
                        arg = less ? (uint32_t)c : arg;
                    }
                }
                word |= arg << (4 * j);
            }
            idx[t] = word;
        }
        // packed tiles of the unit
#pragma unroll
        for (int tt = 0; tt < UC / TK; ++tt) {
            const int kt = col0 / TK + tt;
            const long long tile = ((long long)(rb / p.SB) * p.KT + kt) * p.SB + rb % p.SB;
            uint8_t* base = p.packed + tile * TILE_BYTES;
            const uint32_t* x = idx + tt * STEPS;
            if constexpr (BITS == 4) {
                *reinterpret_cast<u32x4*>(base + 16 * lane) = u32x4{x[0], x[1], x[2], x[3]};
            } else if constexpr (BITS == 2) {
                u32x4 out;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    uint32_t v = 0;
#pragma unroll
                    for (int e = 0; e < 16; ++e) v |= ((x[2 * d + e / 8] >> (4 * (e % 8))) & 3u) << (2 * e);
                    out[d] = v;
                }
                *reinterpret_cast<u32x4*>(base + 16 * lane) = out;
            } else {
                u32x4 lo;
                u32x2 hi;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    uint32_t v = 0;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {                 // byte q: indices 2q, 2q+1 of steps 2d, 2d+1
                        const uint32_t a0 = (x[2 * d] >> (8 * q)) & 3u, a1 = (x[2 * d] >> (8 * q + 4)) & 3u;
                        const uint32_t b0 = (x[2 * d + 1] >> (8 * q)) & 3u, b1 = (x[2 * d + 1] >> (8 * q + 4)) & 3u;
                        v |= (a0 | (a1 << 2) | (b0 << 4) | (b1 << 6)) << (8 * q);
                    }
                    lo[d] = v;
                }
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    uint32_t v = 0;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const uint32_t a = (x[4 * h + u] >> (8 * q + 2)) & 1u, b = (x[4 * h + u] >> (8 * q + 6)) & 1u;
                            v |= (a << (2 * u) | b << (2 * u + 1)) << (8 * q);
                        }
                    hi[h] = v;
                }
                *reinterpret_cast<u32x4*>(base + 16 * lane) = lo;
                *reinterpret_cast<u32x2*>(base + 1024 + 8 * lane) = hi;
            }
        }
    }
}

namespace {

template <int BITS, int GROUP>
hipError_t launch_q(bool wf32, const QuantParams& p, int grid, hipStream_t stream) {
    if (wf32) hipLaunchKernelGGL((quantize_kernel<BITS, GROUP, true>), dim3(grid), dim3(256), 0, stream, p);
    else hipLaunchKernelGGL((quantize_kernel<BITS, GROUP, false>), dim3(grid), dim3(256), 0, stream, p);
    return hipGetLastError();
}

template <int BITS>
hipError_t launch_qb(int group, bool wf32, const QuantParams& p, int grid, hipStream_t stream) {
    switch (group) {
        case 32: return launch_q<BITS, 32>(wf32, p, grid, stream);
        case 64: return launch_q<BITS, 64>(wf32, p, grid, stream);
        case 128: return launch_q<BITS, 128>(wf32, p, grid, stream);
        case 256: return launch_q<BITS, 256>(wf32, p, grid, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace
}  // namespace lutq

extern "C" lutq_status lutq_quantize(const void* W, int w_is_f32, const void* lut, int bits, int group_size,
                                     int64_t N, int64_t K, lutq_dtype dtype, void* scales_out, void* packed_out,
                                     void* stream) {
    if (!W || !lut || !scales_out || !packed_out) return LUTQ_ERR_NULL;
    if (lutq_packed_bytes(N, K, bits, group_size) == 0) {
        if (bits < 2 || bits > 4) return LUTQ_ERR_BITS;
        if ((group_size != 32 && group_size != 64 && group_size != 128 && group_size != 256) ||
            (K > 0 && K % group_size != 0))
            return LUTQ_ERR_GROUP;
        return LUTQ_ERR_SHAPE;
    }
    if (dtype != LUTQ_F16 && dtype != LUTQ_BF16) return LUTQ_ERR_DTYPE;
    if (N > (1 << 24) || K > (1 << 24)) return LUTQ_ERR_SHAPE;
    auto aligned16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
    if (!aligned16(W) || !aligned16(packed_out) || (reinterpret_cast<uintptr_t>(scales_out) & 1u) ||
        (reinterpret_cast<uintptr_t>(lut) & 1u))
        return LUTQ_ERR_ALIGN;
    const int tk = lutq::layout::tile_k(bits);
    const int uc = group_size > tk ? group_size : tk;
    const int64_t nb = N / 16;
    lutq::QuantParams p;
    p.W = W;
    p.lut = static_cast<const uint16_t*>(lut);
    p.scales = static_cast<uint16_t*>(scales_out);
    p.packed = static_cast<uint8_t*>(packed_out);
    p.N = (int)N; p.K = (int)K;
    p.KT = (int)(K / tk);
    p.SG = (int)(K / group_size);
    p.SB = lutq::layout::super_block(nb);
    p.upr = (int)(K / uc);
    p.units = nb * (K / uc);
    p.bf16 = dtype == LUTQ_BF16;
    int64_t grid = (p.units + 3) / 4;
    if (grid > 16384) grid = 16384;
    const hipStream_t s = static_cast<hipStream_t>(stream);
    const hipError_t e = bits == 2 ? lutq::launch_qb<2>(group_size, w_is_f32 != 0, p, (int)grid, s)
                       : bits == 3 ? lutq::launch_qb<3>(group_size, w_is_f32 != 0, p, (int)grid, s)
                                   : lutq::launch_qb<4>(group_size, w_is_f32 != 0, p, (int)grid, s);
    return e == hipSuccess ? LUTQ_OK : LUTQ_ERR_DEVICE;
}
