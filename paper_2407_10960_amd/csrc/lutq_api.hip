// C-ABI entry points of liblutq.so for the device side: argument validation, the choice of work
// decomposition (host part of Algorithm 1: tile scheduler and number of blocks), kernel launch.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <mutex>

#include "lutq.h"
#include "lutq_launch.hpp"

namespace {

using namespace lutq;

constexpr int kMaxGrid = 4096;
constexpr size_t kCounterBytes = 64 * 1024;                                   // 16384 row groups
constexpr size_t kSlotBytes = (size_t)kSlotFloats * sizeof(float);            // 8 KiB
constexpr size_t kWorkspaceBytes = kCounterBytes + (size_t)kMaxGrid * 2 * kSlotBytes;

inline int tile_k(int bits) { return bits == 4 ? 128 : 256; }

lutq_status check_problem(int bits, int group_size, int64_t N, int64_t K) {
    if (bits < 2 || bits > 4) return LUTQ_ERR_BITS;
    if (group_size != 32 && group_size != 64 && group_size != 128) return LUTQ_ERR_GROUP;
    if (N <= 0 || K <= 0 || N % 16 != 0 || K % tile_k(bits) != 0) return LUTQ_ERR_SHAPE;
    if (N / 16 > (int64_t)(kCounterBytes / 4) || N > (1 << 24) || K > (1 << 24)) return LUTQ_ERR_SHAPE;
    // the kernels address every buffer with 32-bit offsets and use offsets >= 2 GiB as "out of range"
    if (N * K * bits / 8 >= (int64_t)1 << 31 || N * (K / 32) * 2 >= (int64_t)1 << 31 || 32 * K * 2 >= (int64_t)1 << 31)
        return LUTQ_ERR_SHAPE;
    if (K % group_size != 0) return LUTQ_ERR_GROUP;
    return LUTQ_OK;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct DeviceInfo {
    int cus = 0;
    bool ok = false;
};

// Number of compute units of the current device (queried once per device).
DeviceInfo device_info() {
    static std::mutex mu;
    static DeviceInfo cache[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return DeviceInfo{};
    std::lock_guard<std::mutex> lock(mu);
    if (!cache[dev].ok) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            return DeviceInfo{};
        cache[dev].cus = cus;
        cache[dev].ok = true;
    }
    return cache[dev];
}

// bytes of the replicated table in LDS of lutq_dequant (8 copies)
inline int super_block(int64_t nb) { return nb % 4 == 0 ? 4 : nb % 2 == 0 ? 2 : 1; }
int lut_bytes(int bits, int log2c) { return (bits == 3 ? 64 * 4 : bits == 4 ? 256 * 4 : 256 * 8) << log2c; }

int ilog2(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

// Default work decomposition (host part of Algorithm 1: the tile scheduler and the number of blocks).
// Tiles = (N / 16R) row groups x (K / TK) K tiles, cut into `grid` equal contiguous ranges.
//
// Measured on MI355X, the cross-workgroup fix-up costs three dependent device-scope round trips
// (store partials, bump the counter, read the slots), several microseconds, which is more than the
// wave quantisation it would remove on these decode shapes.  So the default keeps every output tile
// inside one workgroup whenever that still gives each compute unit a workgroup: R is the largest of
// 4, 2, 1 with at least one row group per compute unit, and grid = number of row groups.  Only when
// N is too small for that (fewer 16-row blocks than compute units) is K split across workgroups,
// into j equal parts per row group, with the Stream-K style fix-up.
lutq_status default_plan(int bits, int group_size, int64_t M, int64_t N, int64_t K, int cus, int force_r,
                         lutq_plan* plan) {
    (void)group_size;
    const int64_t nb = N / 16, kt = K / tile_k(bits);
    int r = super_block(nb);                              // R has to divide the layout's super-block
    while (r > 1 && nb / r < cus) r >>= 1;
    if (force_r) r = force_r;
    const int64_t groups = nb / r;
    int64_t grid = groups;
    if (groups < cus) {
        int64_t j = (cus + groups - 1) / groups;         // K parts per row group
        if (j > kt / 4) j = kt / 4;                      // keep at least one K tile per wavefront
        if (j < 1) j = 1;
        grid = groups * j;
    }
    while (grid > kMaxGrid) grid = (grid + 1) / 2;
    plan->row_blocks_per_wave = r;
    plan->grid = (int)grid;
    plan->waves_per_workgroup = 4;
    plan->tiles_in_flight = (r == 4 && M > 16) ? 2 : 4;
    return LUTQ_OK;
}

typedef hipError_t (*matmul_launcher)(int, int, int, int, int, bool, int, const MatmulParams&, hipStream_t);
typedef hipError_t (*dequant_launcher)(int, const DequantParams&, int, int, hipStream_t);

matmul_launcher pick_matmul(int bits, lutq_dtype dt) {
    if (dt == LUTQ_F16) return bits == 2 ? launch_matmul_b2_F16 : bits == 3 ? launch_matmul_b3_F16 : launch_matmul_b4_F16;
    return bits == 2 ? launch_matmul_b2_BF16 : bits == 3 ? launch_matmul_b3_BF16 : launch_matmul_b4_BF16;
}
dequant_launcher pick_dequant(int bits, lutq_dtype dt) {
    if (dt == LUTQ_F16) return bits == 2 ? launch_dequant_b2_F16 : bits == 3 ? launch_dequant_b3_F16 : launch_dequant_b4_F16;
    return bits == 2 ? launch_dequant_b2_BF16 : bits == 3 ? launch_dequant_b3_BF16 : launch_dequant_b4_BF16;
}

}  // namespace

extern "C" const char* lutq_status_string(lutq_status s) {
    switch (s) {
        case LUTQ_OK: return "ok";
        case LUTQ_ERR_NULL: return "null pointer";
        case LUTQ_ERR_BITS: return "bits must be 2, 3 or 4";
        case LUTQ_ERR_GROUP: return "group_size must be 32, 64 or 128 and divide K";
        case LUTQ_ERR_SHAPE: return "unsupported shape (1 <= M <= 32, N % 16 == 0, K % K-tile == 0)";
        case LUTQ_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case LUTQ_ERR_INDEX_RANGE: return "index out of range for the bit width";
        case LUTQ_ERR_WORKSPACE: return "workspace missing or too small";
        case LUTQ_ERR_DTYPE: return "dtype must be LUTQ_F16 or LUTQ_BF16";
        case LUTQ_ERR_DEVICE: return "HIP runtime error";
        case LUTQ_ERR_PLAN: return "invalid plan";
    }
    return "unknown status";
}

extern "C" size_t lutq_workspace_bytes(int64_t N, int64_t K, int bits, int group_size) {
    if (check_problem(bits, group_size, N, K) != LUTQ_OK) return 0;
    return kWorkspaceBytes;
}

extern "C" lutq_status lutq_plan_default(int bits, int group_size, int64_t M, int64_t N, int64_t K,
                                         lutq_dtype dtype, lutq_plan* plan) {
    if (!plan) return LUTQ_ERR_NULL;
    lutq_status st = check_problem(bits, group_size, N, K);
    if (st != LUTQ_OK) return st;
    if (M < 1 || M > 32) return LUTQ_ERR_SHAPE;
    if (dtype != LUTQ_F16 && dtype != LUTQ_BF16) return LUTQ_ERR_DTYPE;
    DeviceInfo di = device_info();
    if (!di.ok) return LUTQ_ERR_DEVICE;
    return default_plan(bits, group_size, M, N, K, di.cus, 0, plan);
}

extern "C" lutq_status lutq_matmul_plan(const void* X, const void* packed, const void* scales, const void* lut,
                                        int bits, int group_size, int64_t M, int64_t N, int64_t K,
                                        lutq_dtype dtype, void* Y, void* workspace, size_t workspace_bytes,
                                        void* stream, const lutq_plan* user_plan) {
    if (!X || !packed || !scales || !lut || !Y) return LUTQ_ERR_NULL;
    lutq_status st = check_problem(bits, group_size, N, K);
    if (st != LUTQ_OK) return st;
    if (M < 1 || M > 32) return LUTQ_ERR_SHAPE;
    if (dtype != LUTQ_F16 && dtype != LUTQ_BF16) return LUTQ_ERR_DTYPE;
    if (!aligned16(X) || !aligned16(packed) || !aligned16(scales) || !aligned16(Y) || !aligned16(workspace))
        return LUTQ_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(lut) & 1u) != 0) return LUTQ_ERR_ALIGN;
    if (!workspace || workspace_bytes < kWorkspaceBytes) return LUTQ_ERR_WORKSPACE;

    DeviceInfo di = device_info();
    if (!di.ok) return LUTQ_ERR_DEVICE;
    const int64_t nb = N / 16, kt = K / tile_k(bits);
    int force_r = 0;
    if (user_plan) {
        const int w = user_plan->waves_per_workgroup;
        const int f = user_plan->tiles_in_flight;
        if ((w != 0 && w != 4 && w != 8) || (f != 0 && f != 2 && f != 4)) return LUTQ_ERR_PLAN;
        force_r = user_plan->row_blocks_per_wave;
        if (force_r != 0 && ((force_r != 1 && force_r != 2 && force_r != 4) || super_block(nb) % force_r != 0))
            return LUTQ_ERR_PLAN;
    }
    lutq_plan plan;
    default_plan(bits, group_size, M, N, K, di.cus, force_r, &plan);
    if (user_plan) {
        if (user_plan->grid != 0) {
            if (user_plan->grid < 1 || user_plan->grid > kMaxGrid) return LUTQ_ERR_PLAN;
            plan.grid = user_plan->grid;
        }
        if (user_plan->waves_per_workgroup != 0) plan.waves_per_workgroup = user_plan->waves_per_workgroup;
        if (user_plan->tiles_in_flight != 0) plan.tiles_in_flight = user_plan->tiles_in_flight;
    }
    const int r = plan.row_blocks_per_wave;
    const int64_t tiles = (nb / r) * kt;
    if (plan.grid > tiles) plan.grid = (int)tiles;      // every workgroup must own at least one tile

    MatmulParams p;
    p.X = static_cast<const uint16_t*>(X);
    p.packed = static_cast<const uint8_t*>(packed);
    p.scales = static_cast<const uint16_t*>(scales);
    p.lut = static_cast<const uint16_t*>(lut);
    p.Y = static_cast<uint16_t*>(Y);
    p.counters = static_cast<uint32_t*>(workspace);
    p.slots = reinterpret_cast<float*>(static_cast<char*>(workspace) + kCounterBytes);
    p.packed_bytes = (uint32_t)(N * K * bits / 8);
    p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.KT = (int)kt;
    p.NRG = (int)(nb / r);
    p.G = plan.grid;
    p.TQ = (int)(tiles / plan.grid);
    p.TR = (int)(tiles % plan.grid);
    p.SG = (int)(K / group_size);
    p.SBL = ilog2(super_block(nb));
    const int mb = M > 16 ? 2 : 1;
    const bool sch = (K / group_size) % 8 == 0;            // scale rows are 16-byte aligned: chunked scale path
    int nw = plan.waves_per_workgroup, stages = plan.tiles_in_flight;
    if (!sch) { nw = 4; stages = 2; }                      // the per-tile scale path exists in one shape only
    if (!matmul_instance_exists(nw, stages, sch)) return LUTQ_ERR_PLAN;
    // M <= 4: four K steps of activations per load, rotated into place (a quarter of the registers)
    int xm = (M <= 4) ? 4 : 16;
    if (const char* ev = std::getenv("LUTQ_XM")) xm = (std::atoi(ev) == 16 || M > 4) ? 16 : 4;
    hipError_t e = pick_matmul(bits, dtype)(group_size, mb, r, nw, stages, sch, xm, p, static_cast<hipStream_t>(stream));
    if (e != hipSuccess && std::getenv("LUTQ_VERBOSE"))
        std::fprintf(stderr, "lutq_matmul: launch failed: %s (grid %d, block %d)\n", hipGetErrorString(e), p.G, nw * 64);
    return e == hipSuccess ? LUTQ_OK : LUTQ_ERR_DEVICE;
}

extern "C" lutq_status lutq_matmul(const void* X, const void* packed, const void* scales, const void* lut,
                                   int bits, int group_size, int64_t M, int64_t N, int64_t K, lutq_dtype dtype,
                                   void* Y, void* workspace, size_t workspace_bytes, void* stream) {
    return lutq_matmul_plan(X, packed, scales, lut, bits, group_size, M, N, K, dtype, Y, workspace,
                            workspace_bytes, stream, nullptr);
}

extern "C" lutq_status lutq_dequant(const void* packed, const void* scales, const void* lut, int bits,
                                    int group_size, int64_t N, int64_t K, lutq_dtype dtype, void* W_out,
                                    void* stream) {
    if (!packed || !scales || !lut || !W_out) return LUTQ_ERR_NULL;
    lutq_status st = check_problem(bits, group_size, N, K);
    if (st != LUTQ_OK) return st;
    if (dtype != LUTQ_F16 && dtype != LUTQ_BF16) return LUTQ_ERR_DTYPE;
    if (!aligned16(packed) || !aligned16(scales) || !aligned16(W_out)) return LUTQ_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(lut) & 1u) != 0) return LUTQ_ERR_ALIGN;
    DeviceInfo di = device_info();
    if (!di.ok) return LUTQ_ERR_DEVICE;
    DequantParams p;
    p.packed = static_cast<const uint8_t*>(packed);
    p.scales = static_cast<const uint16_t*>(scales);
    p.lut = static_cast<const uint16_t*>(lut);
    p.W = static_cast<uint16_t*>(W_out);
    p.packed_bytes = (uint32_t)(N * K * bits / 8);
    p.N = (int)N; p.K = (int)K;
    p.KT = (int)(K / tile_k(bits));
    p.SG = (int)(K / group_size);
    p.SB = super_block(N / 16);
    p.tiles = (N / 16) * (int64_t)p.KT;
    p.log2c = 3;
    int64_t grid = (p.tiles + 3) / 4;
    const int64_t cap = (int64_t)di.cus * 8;
    if (grid > cap) grid = cap;
    hipError_t e = pick_dequant(bits, dtype)(group_size, p, (int)grid, lut_bytes(bits, p.log2c) + 2048,
                                             static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LUTQ_OK : LUTQ_ERR_DEVICE;
}
