// C-ABI entry points of liblutq.so for the device side: argument validation, the choice of work
// decomposition (host part of Algorithm 1: tile scheduler and number of blocks), kernel launch.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <mutex>
#include <vector>

#include "lutq.h"
#include "lutq_calib.h"
#include "lutq_launch.hpp"
#include "lutq_layout.hpp"

namespace {

using namespace lutq;

constexpr int kMaxGrid = 4096;
constexpr int64_t kMaxRows = 128;                  // activation rows of one call (slices of 32 or 64 per launch)
constexpr size_t kCounterBytes = 64 * 1024;                                   // 16384 row groups
constexpr size_t kSlotBytes = (size_t)kSlotFloats * sizeof(float);            // 8 KiB
constexpr size_t kWorkspaceBytes = kCounterBytes + (size_t)kMaxGrid * 2 * kSlotBytes;

// Scratch of lutq_matmul_static: the same two areas (arrival counters, partial-sum slots) in a device array
// of the library's own, so that the call needs no workspace from the caller and allocates nothing.  Every
// device the library runs on holds its own copy from the moment the code object is loaded until the
// process ends.  Device globals start zeroed, and every launch returns the counters it used to zero, so the
// counters are zero whenever a launch starts; the slots are overwritten before they are read.
constexpr size_t kStaticSlotBytes = LUTQ_STATIC_SCRATCH_BYTES - kCounterBytes;
static __device__ __align__(256) unsigned char scratch[LUTQ_STATIC_SCRATCH_BYTES];

// the operand-order copy of the activations for row-streaming launches beyond 32 rows (XopParams)
__global__ __launch_bounds__(256) void rows_xop_kernel(const XopParams p) {
    const int kt = (int)blockIdx.x, mb = (int)blockIdx.y;   // one workgroup per (K tile, block of sixteen rows)
    const int chunks = p.STEPS * 4;                       // 16-byte chunks per row of a tile
    for (int i = (int)threadIdx.x; i < 16 * chunks; i += 256) {
        const int li = i / chunks, c = i - li * chunks;
        const int m = 16 * mb + li;
        u32x4 v = u32x4{0u, 0u, 0u, 0u};
        if (m < p.M) v = *reinterpret_cast<const u32x4*>(p.X + (size_t)m * p.K + (size_t)kt * (chunks * 8) + 8 * c);
        const int s = c >> 2, lo = c & 3;
        *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(p.Xop) + ((size_t)((kt * p.STEPS + s) * p.MB + mb) * 64 + (lo * 16 + li)) * 16) = v;
    }
}

using layout::super_block;
using layout::tile_k;

lutq_status check_problem(int bits, int group_size, int64_t N, int64_t K) {
    if (bits < 2 || bits > 4) return LUTQ_ERR_BITS;
    if (group_size != 32 && group_size != 64 && group_size != 128 && group_size != 256) return LUTQ_ERR_GROUP;
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

// bytes of lutq_dequant's table (log2c copies); entries are 8 bytes for the 2-bit quad table and for the
// widened bf16 pair tables, else 4
int lut_bytes(int bits, bool bf16, int log2c) {
    return ((bits == 3 ? 64 : 256) * ((bits == 2 || bf16) ? 8 : 4)) << log2c;
}

int ilog2(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

// Everything the launch needs to know about the work decomposition.
struct Decomp {
    int r, grid, nw, stages, rs;      // the first five plan fields, all chosen
    int queue = 0;                    // work-queue kernel (M <= 4): rs = row groups per workgroup, it = tiles per item
    int it = 0;
    int rows = 0;                     // row-streaming kernel: r = row blocks side by side, rs = row blocks per workgroup
    int ks = 0;                       // ... K slices across workgroups (0, 1: none): grid = shares x ks, it = K tiles per slice
};

int rows_table_bytes(int bits) { return bits == 2 ? lut_row_table_bytes<2>() : bits == 3 ? lut_row_table_bytes<3>() : lut_row_table_bytes<4>(); }
// waves the row-streaming instance (bits, dtype, M half count, row blocks side by side) is compiled for; 0 = none
int rows_instance_waves(int bits, bool bf16, int mb, int amax) {
    const bool wide = bf16 ? (bits == 2 ? Tab<2, BF16>::WIDE : bits == 3 ? Tab<3, BF16>::WIDE : Tab<4, BF16>::WIDE)
                           : (bits == 2 ? Tab<2, F16>::WIDE : bits == 3 ? Tab<3, F16>::WIDE : Tab<4, F16>::WIDE);
    return (amax == 4 || amax == 8) ? rows_max_waves(bits, mb, amax, wide) : 0;
}

// Row-streaming decomposition (rows_kernel): one workgroup per compute unit (per row block where there
// are fewer), whole row blocks each, eight row blocks side by side where the instance exists, as many
// waves as it was compiled for (no more than K tiles).
// LDS offset of the row-streaming kernel's reduction slots (behind the table and the scales of `side` row
// blocks), and how many row blocks one round of the reduction can hold (0: the launch does not fit)
// (tab16 > 0: one table per output row -- `side` sixteen-copy tables of tab16 bytes and their raw rows instead of
// the shared table)
int rows_red_off(int bits, int side, int sg2, int tab16 = 0) {
    const int tables = tab16 > 0 ? side * (tab16 + 16 * (1 << bits) * 2) : rows_table_bytes(bits);
    return tables + side * 16 * (sg2 + 16);
}
int rows_blocks_per_round(int bits, int side, int sg2, int mb, int nw, int tab16 = 0) {
    const int room = 160 * 1024 - rows_red_off(bits, side, sg2, tab16);
    return room <= 0 ? 0 : room / (mb * nw * 1024);
}

bool rows_decomp(int bits, bool bf16, int64_t M, int64_t N, int64_t K, int group_size, int cus, Decomp* out) {
    const int64_t nb = N / 16, kt = K / tile_k(bits);
    const int mb = M > 16 ? 2 : 1;
    const int grid = (int)(nb < cus ? nb : cus);
    const int64_t per = nb / grid;
    if (per > 64) return false;
    int amax = per + (nb % grid ? 1 : 0) > 4 ? 8 : 4;
    int nw = rows_instance_waves(bits, bf16, mb, amax);
    if (nw == 0) { amax = 4; nw = rows_instance_waves(bits, bf16, mb, amax); }
    if (nw == 0) return false;
    if (nw > kt) nw = (int)(kt < 4 ? 4 : kt);
    if (rows_blocks_per_round(bits, amax, (int)(K / group_size) * 2, mb, nw) < 1) return false;
    out->r = amax; out->grid = grid; out->nw = nw; out->stages = 2; out->rs = (int)per; out->queue = 0; out->it = 0; out->rows = 1;
    return true;
}

// Where the row-streaming kernel is the default (M >= 5).  Measured against the team plans on the gate+up and
// QKV shapes of LLaMA-2-7B/13B and LLaMA-3-8B/70B, M = 8, 16, 24, 32, fp16 and bf16, MI355X:
//   * 4 bits, five to eight row blocks per compute unit (one pass), M > 8: 3-10 % faster where the row blocks
//     do not divide over the compute units (7B gate+up M = 16: 15.8 -> 14.2 us, bf16 18.1 -> 16.3; 13B: 20.5 ->
//     18.9); where they do (8B gate+up) 1-6 % in bf16 (M = 16: 18.4 -> 17.3 us), 1.5 % in fp16 up to sixteen rows
//     (16.0 -> 15.7, 16.5 -> 16.2 us in two runs) and within the noise of either beyond, which stays with the teams.  With more (70B gate+up, fourteen: two passes, each with its own
//     ramp and reduction) the teams are faster, and at M <= 8 they are as fast.
//   * 3 bits, the same shapes, 8 < M <= 16: 6-19 % (13B gate+up 20.5 -> 17.8 us, bf16 24.3 -> 19.7).
//   * 4 bits, two to four row blocks per compute unit that do not divide (QKV shapes), M <= 16, bf16 M <= 24:
//     70B QKV M = 8 14.2 -> 13.3 us, M = 16 17.5 -> 16.2, bf16 M = 24 23.2 -> 20.4; beyond that the teams win.
bool default_rows_decomp(int bits, bool bf16, int64_t M, int64_t N, int64_t K, int group_size, int cus, Decomp* out) {
    if (M < 5 || ((K / group_size) * 2) % 16 != 0) return false;
    const int64_t nb = N / 16;
    if (nb < cus) return false;
    const int64_t per = nb / cus;
    const bool uneven = nb % cus != 0;
    const int64_t amax = per + (uneven ? 1 : 0);
    bool take = false;
    // Three to four row blocks per compute unit (QKV of LLaMA-2-7B and 13B, not in the benchmark), 3-bit or bf16, up
    // to 24 rows: 7B QKV bf16 M = 16 12.1 -> 9.9 us, 3-bit M = 16 11.7 -> 10.3, M = 24 16.8 -> 13.1; 13B QKV 3-bit M = 8
    // 15.4 -> 11.8, M = 24 22.3 -> 17.2; in fp16 at 4 bits the two kernels are within 3 % there, and with two per
    // compute unit (70B O) the teams win.
    const bool few = per >= 3 && amax <= 4 && M <= 24 && (bits == 3 || bf16);
    if (bits == 4) take = (per >= 5 && amax <= 8 && M > 8 && (uneven || bf16 || M <= 16)) || (uneven && per >= 2 && amax <= 4 && M <= (bf16 ? 24 : 16)) || few;
    // (3 bits from six row blocks per compute unit: from five rows up -- 13B gate+up M = 6 / 8 24.8 / 25.3 -> 16.5 / 17.1 us,
    // 8B gate+up M = 8 15.6 -> 15.2; with five to six per unit, 7B gate+up, the teams are faster up to eight rows)
    else if (bits == 3) take = (per >= 5 && amax <= 8 && M > 8 && M <= 16) || (per >= 6 && amax <= 8 && M <= 16) || few;
    // (only where one pass covers the workgroup's row blocks: a second pass costs more than the teams)
    return take && rows_decomp(bits, bf16, M, N, K, group_size, cus, out) && out->r >= amax;
}

// K slices on the row-streaming kernel (9..32 rows): for matrices with at most one row block per compute
// unit (two up to 24 rows) and a long K, four row blocks per share of workgroups and as many K slices as keep the grid within the compute
// units, at least three slices of at least 1792 columns (fourteen 4-bit K tiles) each, as even as whole tiles allow; every workgroup then reads only its slice of the activations with eight (twelve) waves
// that hold them in registers, and a share's slices are added by whichever of its workgroups finishes last.  Measured against the team plans (MI355X, us,
// HBM-cold weights): 8B down (4096 x 14336) M = 17 / 24 / 32 20.1 / 20.1 / 20.5 -> 14.5 / 15.4 / 16.8, bf16 M = 32 21.3 -> 16.9,
// 3-bit 21.2 -> 17.9, group 32 20.5 -> 17.9; 4096 x 8192 M = 20 / 32 13.2 / 15.2 -> 11.3 / 12.5; 4096 x 28672 31.8 -> 26.4;
// 2048 x 14336 18.9 -> 13.0; 3072 x 12288 24.0 -> 15.9; M = 12 / 16: 8B down 12.3 / 13.4 -> 12.1 / 12.6 (bf16 M = 16 14.3 -> 13.0, 3-bit
// 14.6 -> 13.7), 4096 x 28672 19.8 / 21.8 -> 17.5 / 18.5, 3072 x 12288 14.5 / 15.3 -> 10.7 / 11.3, 2048 x 14336 10.5 / 11.6 -> 10.2 / 10.6.
// M = 9..11: 70B down bf16 35.0-37.1 -> 29.5-30.0, 3072 x 12288 M = 10 13.6 -> 10.4, 4096 x 28672 M = 9 17.9 -> 17.0, 8B down level to 5 %.
// 2 bits: 8B down M = 16 / 24 / 32 12.9 / 20.2 / 20.7 -> 11.9 / 15.2 / 16.6 (bf16 M = 32 22.8 -> 17.9), 4096 x 28672 M = 16 / 32 22.5 / 26.7 -> 16.2 / 24.9,
// 3072 x 12288 M = 20 19.2 -> 13.2, 2048 x 14336 M = 32 19.2 -> 15.7.
// Not taken: below nine rows (M = 8: 2 % faster to 11 % slower), slices of eight tiles
// (8B O: 10.8 -> 10.2 at M = 32 but 9.3 -> 10.0 at M = 24), grids below half the compute units (1024 x 8192: 11.0 -> 12.3),
// fewer than four slices (8B O in two slices of sixteen tiles: M = 20 8.6 -> 9.7), more than one row block per compute unit
// (8B QKV, 70B O and down, N = K = 8192: within 3 % either way).
bool sliced_rows_decomp(int bits, bool bf16, int64_t M, int64_t N, int64_t K, int group_size, int cus, Decomp* out) {
    if (M < 9 || M > 32) return false;
    const int64_t nb = N / 16, kt = K / tile_k(bits);
    const int mb = M > 16 ? 2 : 1;
    if (nb > 2 * (int64_t)cus || nb % 4 != 0) return false;
    const int64_t shares = nb / 4;
    // (three slices like four: 13B down, 5120 x 13824, 80 shares x 3 slices on 240 units, M = 12 / 16 / 24 / 32 19.1 / 20.0 / 26.3 /
    // 29.3 -> 14.1 / 14.9 / 17.6 / 19.4 us, the same at 2 and 3 bits and in bf16; 7B down, 4096 x 11008, in slices of 22, 22, 21, 21
    // tiles: M = 32 19.1 -> 15.9)
    // (three slices up to sixteen rows only from 4096 columns each: 4096 x 6144 M = 12 8.0 -> 9.2 us, but M = 24 12.5 -> 11.3)
    // (two slices only at 4 bits up to 24 rows and with slices of 56 tiles or more -- two row blocks per compute
    // unit and a long K, 70B down: bf16 M = 9 / 12 / 16 / 20 / 24 35.0 / 37.9 / 35.0 / 41.6 / 41.7 -> 29.5 / 30.2 / 31.6 / 39.0 / 39.7 us,
    // fp16 M = 16 / 20 32.1 / 39.2 -> 30.6 / 36.8; at M = 32 43.0 -> 43.8; on K = 8192 -- 70B O, N = K = 8192 -- within 5 % either
    // way, and at 3 bits the teams are 1-5 % faster)
    int ks = 0;
    // (only slice counts that a plan can name: k = the K tiles divided by the tiles per slice, rounded up)
    auto nameable = [&](int64_t k) { const int64_t it = (kt + k - 1) / k; return (kt + it - 1) / it == k; };
    for (int64_t k = cus / shares; k >= 2 && !ks; --k)
        if (!nameable(k)) continue;
        else if (k >= 3 ? kt / k * tile_k(bits) >= (k == 3 && mb == 1 ? 4096 : 14 * 128) : kt / k >= 56 && bits == 4 && M <= 24) ks = (int)k;
    // (grids from half the compute units up beyond sixteen rows, from three quarters up to there: 2048 x 8192 on 128
    // workgroups M = 24 11.9 -> 11.0 us, but bf16 M = 16 9.1 -> 10.0)
    if (!ks || shares * ks * (mb == 2 ? 2 : 4) < cus * (mb == 2 ? 1 : 3) || shares * 64 > (int64_t)kCounterBytes) return false;
    // (eight waves beyond sixteen rows, twelve up to there: 8B down M = 16 13.1 / 12.5 / 12.8 us with 8 / 12 / 16)
    int nw = rows_instance_waves(bits, bf16, mb, 4);
    if (nw > (mb == 2 ? 8 : 12)) nw = mb == 2 ? 8 : 12;
    if (nw < 4 || rows_blocks_per_round(bits, 4, (int)(K / group_size) * 2, mb, nw) < 1) return false;
    out->r = 4; out->grid = (int)(shares * ks); out->nw = nw; out->stages = 2; out->rs = 4; out->queue = 0;
    out->it = (int)((kt + ks - 1) / ks); out->ks = ks; out->rows = 1;
    return true;
}

// 33..64 activation rows in one pass over the weights: the row-streaming kernel with three or four M blocks
// (4 bits, scale rows of whole 16-byte units, four row blocks side by side, activations from their
// operand-order copy).  `take`: whether that is also the default (against two launches of 32 rows).
bool wide_rows_decomp(int bits, bool bf16, int64_t M, int64_t N, int64_t K, int group_size, int cus, Decomp* out, bool* take) {
    if (M <= 32 || M > 64) return false;
    const int64_t nb = N / 16, kt = K / tile_k(bits);
    const int mb = (int)((M + 15) / 16);
    const int grid = (int)(nb < cus ? nb : cus);
    const int64_t per = nb / grid;
    if (per > 64) return false;
    int nw = rows_instance_waves(bits, bf16, mb, 4);
    if (nw == 0) return false;
    if (nw > kt) nw = (int)(kt < 4 ? 4 : kt);
    if (rows_blocks_per_round(bits, 4, (int)(K / group_size) * 2, mb, nw) < 1) return false;
    out->r = 4; out->grid = grid; out->nw = nw; out->stages = 2; out->rs = (int)per; out->queue = 0; out->it = 0; out->rows = 1;
    // Measured against two launches of 32 rows (MI355X, M = 64, us): 8B QKV 23.6 -> 16.6, O 21.5 -> 14.9, gate+up 42.3 ->
    // 32.1 (bf16 46.4 -> 32.7), down 40.4 -> 33.9; 70B QKV bf16 46.7 -> 28.1, O 37.6 -> 25.9, gate+up 135.7 -> 102.3, down
    // 83.0 -> 71.7; N = K = 8192 group 32 36.5 -> 26.3.  Below one row block per compute unit it was not measured.
    *take = nb >= (int64_t)cus;
    return true;
}

// LDS bytes of a work-queue launch
int queue_lds_bytes(int bits, int nw, int items, int r) {
    return bits == 2 ? decode_lds_bytes<2>(nw, items, r) : bits == 3 ? decode_lds_bytes<3>(nw, items, r) : decode_lds_bytes<4>(nw, items, r);
}

// Work-queue decomposition for M <= 4 (decode_kernel): every workgroup owns `a` row groups of `r` row
// blocks over the whole of K, one workgroup per compute unit, so no partial sum crosses workgroups and
// the queue evens out the waves.  Chosen where it measured faster than the team plans (LLaMA-3 8B and 70B
// shapes, 2/3/4 bits, both dtypes, M = 1 and 4): from eight row blocks per compute unit up at every bit
// width (2-10 %: 70B gate+up 4-bit fp16 42.3 -> 40.8 us, bf16 49.0 -> 45.3, 3-bit 40.8 -> 39.5, 2-bit 30.9 ->
// 28.1); with two row blocks per compute unit for 4-bit weights, M <= 2 and a long K (70B down 22.4 -> 21.4
// us; at 2 and 3 bits, at M = 4 and on the 8192-column O projection the team plans are as fast or faster).
// Seven row blocks per compute unit (8B gate+up: 12.35 against 12.17 us, and 13.8 against 12.6 us at M = 4,
// where an odd count rules out two row blocks per wave) and one (no more items than waves, nothing to
// even out) stay with the teams.
// Returns false when this problem is left to the team plans (or cannot run on the work-queue kernel).
bool queue_decomp(int bits, bool bf16, bool sch, int64_t M, int64_t N, int64_t K, int cus, bool only_if_preferred, Decomp* out) {
    if (M > 4 || !sch) return false;
    const int64_t nb = N / 16, kt = K / tile_k(bits);
    const int64_t per = nb / cus;                      // row blocks per workgroup (the first nb % cus get one more)
    const bool even = nb % cus == 0;
    if (per < 1 || per >= 64) return false;
    // Row blocks that do not divide over the compute units (4-bit, M <= 2; measured against the team plans,
    // which then cut every tile across two workgroups or leave compute units idle): 2.5 per compute unit
    // (70B QKV: 12.2 -> 11.4 us, bf16 13.3 -> 12.6) and more than four (LLaMA-2-7B gate+up, 5.4 per compute
    // unit: 12.0 -> 11.1 us; 13B gate+up, 6.75: 15.3 us either way).  With 1.5 (8B QKV) or 3.75 (13B QKV) per
    // compute unit, at 3 bits and at M = 4 the team plans are as fast or faster.
    // A sweep over the LLaMA-2-7B/13B shapes (not in the benchmark) added: more than four per compute unit also at
    // M = 3, 4, with twelve waves there (7B gate+up M = 4 12.3 -> 11.4 us, bf16 14.7 -> 12.6; 13B gate+up bf16 18.8 -> 17.3);
    // three or more in bf16 (13B QKV bf16 M = 1 11.0 -> 10.4-10.6 us, M = 4 11.4 -> 10.9); and between one and two per
    // compute unit with a short K, where the compute units that get two row blocks deal sixteen or more items to
    // sixteen waves (13B O M = 1 6.3 -> 6.0 us, bf16 6.75 -> 6.3; 8B QKV 5.82 -> 5.73, bf16 M = 4 6.34 -> 6.10).
    const bool uneven_one = !even && per == 1 && bits == 4 && kt % 4 == 0 && kt / 4 <= 16;
    // (with eight or more per compute unit the M = 3, 4 cases stay with the teams: a 128256-row output head and Qwen-72B
    // gate+up, 31 and 14 per unit, are 6 % faster there)
    const bool uneven_preferred = bits == 4 && (((nb * 2) % cus == 0 ? per >= 2 && M <= 2 : per >= 4 && (M <= 2 || per < 8)) ||
                                                (bf16 && per >= 3 && (M <= 2 || per < 8)) || uneven_one);
    // One row block per compute unit with a short K (4-bit, at most eight items of four tiles: 8B O 4.52 -> 4.38
    // us at M = 1, 4.72 -> 4.57 at M = 4): one item per wave, so the queue is never used, but the short set-up
    // of this kernel shows.  A longer K (8B down) is faster with the teams' even static split.
    const bool short_k = even && per == 1 && bits == 4 && kt % 4 == 0 && kt / 4 <= 8;
    // Four to seven row blocks per compute unit at 2 and 3 bits, twelve waves (8B gate+up, seven: 3-bit 13.2 -> 12.1 us,
    // bf16 15.1 -> 13.8, 2-bit 9.7 -> 9.0, M = 4 14.5 -> 13.8; with fourteen or sixteen waves the queue loses to the
    // teams here, and at 4 bits the two are equal: 12.5 against 12.3 us).
    // At 4 bits the same up to two rows and in bf16 (M = 1 12.8 -> 12.4 us, M = 2 13.2 -> 12.6, bf16 15.4 -> 14.4; fp16 M = 4
    // equal).
    const bool few_bits_mid = even && per >= 4 && per < 8 && (bits < 4 || M <= 2 || bf16);
    // Two row blocks per compute unit at 2 bits, and at 3 bits up to two rows, twelve waves (N = K = 8192 group 32, 2-bit:
    // M = 1 7.3 -> 7.1 us, M = 2 7.8 -> 7.3, M = 4 9.0 -> 8.3, bf16 9.5 -> 9.1; 70B O 3-bit bf16 9.9 -> 9.3; sixteen waves: 7.8).
    const bool few_bits_two = even && per == 2 && (bits == 2 || (bits == 3 && M <= 2)) && kt % 4 == 0;
    if (only_if_preferred && !(even ? (per >= 8 || short_k || few_bits_mid || few_bits_two || (per == 2 && bits == 4 && M <= 2 && K >= 16384)) : uneven_preferred)) return false;
    const int sb = super_block(nb);
    // two row blocks per wave halve the activation and scale-chunk loads per weight; 3-bit tiles (two
    // bit-slices) run faster one at a time, and two row blocks per compute unit make more items as R = 1
    const int r = (even && per >= 4 && bits != 3 && per % 2 == 0 && sb % 2 == 0 && decode_instance_exists(bits, bf16, 2)) ? 2 : 1;
    const int64_t a = per / r, amax = a + (even ? 0 : 1);
    // items: at least two tiles (the pipeline depth); four where K allows, eight when that still leaves
    // every wave about four items, so that an item's fold and hand-over stay a small part of its work
    int it = kt % 4 == 0 ? 4 : 2;
    if (kt % 8 == 0 && a * (kt / 8) >= 64 && !few_bits_two) it = 8;
    // Uneven shares of two and three row blocks (70B QKV): items of eight tiles, and sixteen waves in bf16 (M = 1 fp16 11.3 ->
    // 11.0 us, bf16 12.4 -> 11.7; M = 2 11.45 -> 11.3, bf16 12.55 -> 12.0; sixteen waves in fp16: 11.25)
    const bool shares_2_3 = !even && per == 2 && !uneven_one && kt % 8 == 0 && kt / 8 >= 8;
    if (shares_2_3) it = 8;
    if (kt % it != 0) return false;
    int64_t items = amax * (kt / it);
    while (queue_lds_bytes(bits, 16, (int)items, r) > 160 * 1024 && kt % (it * 2) == 0) { it *= 2; items = amax * (kt / it); }
    int nw = items >= 16 ? (((amax <= 3 && !even && !uneven_one) && !(shares_2_3 && bf16)) || few_bits_mid || few_bits_two || (!even && per >= 4 && M > 2) ? 12 : 16)
                         : (int)(items < 4 ? 4 : items);
    if (queue_lds_bytes(bits, nw, (int)items, r) > 160 * 1024) return false;
    out->r = r; out->grid = cus; out->nw = nw; out->stages = 2; out->rs = (int)a; out->queue = 1; out->it = it;
    return true;
}
// Work-queue kernel with one table per output row (M <= 4): the sixteen-copy tables of all of a workgroup's row
// blocks are resident at once, so the number of row blocks per workgroup is what LDS holds (4-bit fp16: eight
// at 16 KiB each); one workgroup per compute unit where that fits, else the smallest multiple of the compute
// units that does (the workgroups of one unit then run one after the other), one workgroup per row block when
// there are fewer than two per unit.
int rowlut16_table_bytes(int bits, bool bf16) {
    return bf16 ? (bits == 2 ? rowlut16_bytes<2, BF16>() : bits == 3 ? rowlut16_bytes<3, BF16>() : rowlut16_bytes<4, BF16>())
                : (bits == 2 ? rowlut16_bytes<2, F16>() : bits == 3 ? rowlut16_bytes<3, F16>() : rowlut16_bytes<4, F16>());
}
int rowlut16_stage(int bits) { return 16 * (1 << bits) * 2; }
int rowlut_queue_lds(int bits, bool bf16, int amax, int nw, int items) {
    const int slots = items * 256, stage = amax * rowlut16_stage(bits);
    return amax * rowlut16_table_bytes(bits, bf16) + 256 + nw * 1024 + (slots > stage ? slots : stage);
}
bool rowlut_queue_decomp(int bits, bool bf16, bool sch, int64_t M, int64_t N, int64_t K, int cus, Decomp* out) {
    if (M > 4 || !sch) return false;
    const int64_t nb = N / 16, kt = K / tile_k(bits);
    const int it = kt % 4 == 0 ? 4 : 2;
    if (kt % it != 0) return false;
    for (int mult = 1; mult <= 16; ++mult) {
        const int64_t grid = nb < 2 * (int64_t)cus ? nb : (int64_t)cus * mult;
        if (grid > nb || grid > kMaxGrid) return false;
        const int64_t a = nb / grid, amax = a + (nb % grid ? 1 : 0);
        const int64_t items = amax * (kt / it);
        const int nw = items >= 16 ? 16 : (int)(items < 4 ? 4 : items);
        if (items <= 4096 && amax * (rowlut16_stage(bits) / 4) <= 2 * nw * 64 &&
            rowlut_queue_lds(bits, bf16, (int)amax, nw, (int)items) <= 160 * 1024) {
            out->r = 1; out->grid = (int)grid; out->nw = nw; out->stages = 2; out->rs = (int)a; out->queue = 1; out->it = it;
            return true;
        }
        if (nb < 2 * (int64_t)cus) return false;
    }
    return false;
}
bool default_queue_decomp(int bits, bool bf16, bool sch, int64_t M, int64_t N, int64_t K, int cus, Decomp* out) {
    return queue_decomp(bits, bf16, sch, M, N, K, cus, true, out);
}

inline int steps_per_tile(int bits) { return bits == 4 ? 4 : 8; }
// Activations can be shared through LDS when the teams are enough to stage a tile's pieces between them.
inline bool teams_can_share_x(int bits, int mb, int rs) { return rs * kXPiecesPerWave >= steps_per_tile(bits) * mb; }
// pieces of a tile each wave stages: one when there are as many teams as pieces, else two
inline int x_pieces_per_wave(int bits, int mb, int rs) { return rs >= steps_per_tile(bits) * mb ? 1 : 2; }

// Environment switches, read once per process.  LUTQ_VERBOSE=1 prints every launch shape and the tuner's
// finalists to stderr (2: also the tuner's first-pass times); LUTQ_NO_SHARED_X=1 and LUTQ_NO_XM8=1 switch
// off the activations shared through LDS and the packed activation loads for M = 5..8 (for comparisons).
struct EnvSwitches {
    int verbose;
    bool no_shared_x, no_xm8;
};
const EnvSwitches& env_switches() {
    static const EnvSwitches e = [] {
        EnvSwitches v{};
        const char* s = std::getenv("LUTQ_VERBOSE");
        v.verbose = !s ? 0 : (s[0] == '2' ? 2 : 1);
        v.no_shared_x = std::getenv("LUTQ_NO_SHARED_X") != nullptr;
        v.no_xm8 = std::getenv("LUTQ_NO_XM8") != nullptr;
        return v;
    }();
    return e;
}

bool wide_exists(int bits, bool bf16, int r, int mb, int stages, int xm) {
    return matmul_instance_exists(bits, bf16, r, mb, stages, true, xm, true);
}

int64_t gcd64(int64_t a, int64_t b) {
    while (b) { const int64_t t = a % b; a = b; b = t; }
    return a;
}

// Default work decomposition (host part of Algorithm 1: the tile scheduler and the number of blocks).
//
// Measured on MI355X, a launch of this kernel is a few microseconds of fixed latencies (argument
// fetch, first HBM round trip, table build, final reduction) around a streaming phase that runs at
// HBM speed, and the cross-workgroup fix-up costs three more dependent device-scope round trips.
// What matters is therefore that every compute unit streams the same number of bytes, that one
// workgroup (one table build) per compute unit does all of it with about 24 KiB or more of weights
// in flight, and that partial sums leave the workgroup only when the kernel is long enough to hide it.
//   * N/16 = per x CUs: one workgroup per compute unit, arranged as RS teams x KS waves, per = RS x R.
//     No output tile is split across workgroups.
//   * 4-bit, N/16 = (p/2) x CUs with small p and at least 96 KiB per compute unit: RS = p row blocks
//     side by side, one workgroup per compute unit, every super-group's K range cut into q parts
//     (Stream-K fix-up for every tile, but perfectly balanced).
//   * otherwise one workgroup of 8 waves per row group, R the largest of 4, 2, 1 that still gives
//     every compute unit a row group; only when N is too small even for that is K split across
//     workgroups, with the fix-up.
Decomp default_decomp(int bits, bool bf16, bool sch, int64_t M, int64_t N, int64_t K, int cus, int force_r, int group_size,
                      bool small_scratch = false) {
    const int64_t nb = N / 16, kt = K / tile_k(bits);
    const int mb = M > 16 ? 2 : 1, xm = M <= 4 ? 4 : 16;
    const int sb = super_block(nb);
    const int64_t g = gcd64(nb, cus), pn = nb / g, qn = cus / g;     // nb / cus = pn / qn
    const int64_t bytes_per_cu = N * K * bits / 8 / cus;
    Decomp d;
    d.stages = 2;                                         // measured: deeper prefetch does not pay at 8-16 waves
    // waves for `rs` teams of `r` row blocks: enough for 24 KiB in flight (r KiB per tile, two tiles
    // per wave), at least 8, at most 16, a multiple of rs, two K tiles or more per wave
    const int max_nw = sch ? 16 : 8;                      // the per-tile scale path has no 16-wave build
    auto waves_for = [&](int r, int64_t rs, int64_t tiles_per_team) -> int {
        int ks = 1;
        while ((int64_t)rs * (ks + 1) <= max_nw && tiles_per_team / (ks + 1) >= 2 &&
               (rs * ks < 8 || rs * ks * r * 2 < 24)) ++ks;
        if (rs == 1 && r == 1 && bits == 4) {
            // one row block per workgroup, its K range split over the waves (measured, 4-bit): eight
            // waves when the whole row block is 32 KiB or less (launching and joining more waves costs
            // more than they gain), fourteen when they divide a long K evenly, else twelve
            if (tiles_per_team <= 32) ks = 8;
            else if (tiles_per_team >= 96 && tiles_per_team % 14 == 0 && max_nw >= 14) ks = 14;
        }
        int nw = (int)rs * ks;
        if (nw > 8 && !wide_exists(bits, bf16, r, mb, 2, xm)) {          // too many registers for more than 8 waves
            ks = (int)(8 / rs);
            nw = (int)rs * ks;
        }
        while (nw < 4 && ks > 0) { ++ks; nw = (int)rs * ks; }     // the table build needs four waves
        return nw;
    };
    if (M > 4) {
        // More than four activation rows: next to its weights every wave needs the M x TK activations
        // of each tile it works on, as many bytes as the weights of M / (4 bits) row blocks (from nine
        // rows up the plain layout pads that to 16 or 32 rows; five to eight rows are loaded packed
        // unless the teams share them through LDS).  The rules below were fitted to timings of all candidate plans
        // (lutq_tune) on the LLaMA-3 8B and 70B layer shapes at M = 8, 16, 32 and 2, 3, 4 bits; they
        // stay within a few per cent of the fastest plan there.
        //
        // Plain plan: one workgroup per row group, the largest R that still fills 60 % of the compute
        // units (or, from nine rows up, half of them when K is long enough to be cut in two); K cut across workgroups
        // when there are too few row groups; four waves (one per SIMD) from M = 13 up.
        auto r_fills = [&](int r) {
            const int64_t groups = nb / r;
            // (3 bits below the team plans' M, and 2 bits up to eight rows with a short K: four row blocks
            // per wave only on one and a half row groups per compute unit or more -- 12288x4096 and
            // 15360x5120 at 3 bits, M = 8: R = 4 11.3 and 14.5 us, R = 2 9.5 and 11.6 us; M = 12: 12.2 and
            // 15.2 us against 10.8 and 13.1 us)
            if (r == 4 && bits < 4 && (bits == 3 ? M <= 15 : (M <= 8 && K < 8192)) && groups < (int64_t)cus * 3 / 2) return false;
            if (groups >= (int64_t)cus * 6 / 10) return true;
            // (up to eight rows load their activations packed, two K steps per load: sharing them
            // between row blocks then no longer repays a K cut -- 4096x14336 at M = 8: 12.1 -> 10.8 us)
            const int64_t j = (cus + groups - 1) / groups;
            // (2 and 3 bits need longer halves: 4096x11008, M = 12, 3 bits: cut 16.5 us, uncut R = 1 11.9 us,
            // while 4096x14336 is faster cut at every bit width)
            return M > 8 && j <= 2 && K / j >= (bits == 4 ? 4096 : 6144);
        };
        int r = force_r;
        if (!r) {
            r = sb;
            while (r > 1 && !r_fills(r)) r >>= 1;
            while (r > 1 && !matmul_instance_exists(bits, bf16, r, mb, 2, true, xm, false)) r >>= 1;   // registers
            // (bf16 3-bit, up to eight rows, short K: half as many row blocks per wave while that leaves at
            // most three row groups per compute unit -- 12288x4096 M = 6 10.2 -> 9.0 us, 5120x5120 9.0 -> 8.0 us)
            if (bits == 3 && bf16 && M <= 8 && r > 1 && K < 8192 && nb / (r / 2) <= (int64_t)cus * 3) r >>= 1;
        }
        const int64_t groups = nb / r;
        int64_t grid = groups;
        // (a cut must repay its fix-up: row groups of 64 KiB or more; from 17 rows up smaller ones too, in two
        // parts -- 1024x4096 at M = 32: 10.4 -> 9.1 us)
        const bool big_groups = (int64_t)r * 16 * K * bits / 8 >= 64 * 1024;
        if (groups < (int64_t)cus * 6 / 10 && (big_groups || M > 16)) {
            int64_t j = (cus + groups - 1) / groups;      // K parts per row group
            if (!big_groups && j > 2) j = 2;
            if (j > kt / 8) j = kt / 8;
            if (j < 1) j = 1;
            grid = groups * j;
        } else if (groups < cus && K >= 12288 && (bits == 4 ? M > 8 : M > 16)) {
            // long K (2 and 3 bits: from 17 rows up; 5120x13824 at 3 bits: M = 12 19.4 us split, 17.6 us not;
            // M = 32 29.4 us split, 32.3 us not): every compute unit takes an equal share of the tiles (not up to eight rows, where
            // the fix-up of every tile costs more than the idle units: 5120x13824 at M = 8, 160 row
            // groups: 17.1 us against 15.8 us uncut)
            grid = cus;
        }
        while (grid > kMaxGrid) grid = (grid + 1) / 2;
        d.r = r; d.grid = (int)grid; d.rs = 1;
        // (2 and 3 bits, up to eight rows, exactly one row group per compute unit: four waves too -- 8192^2 2-bit M = 8 11.6 -> 9.8 us,
        // 8B O and down 3-bit M = 8 2-3 %)
        d.nw = (M > 12 || (r == 4 && groups > cus) || (bits < 4 && (groups > cus || (groups == cus && M <= 8)))) ? 4 : 8;
        // The waves of a workgroup split its K tiles evenly (a row group's, or its part of them where K is cut evenly
        // across workgroups); a split that also falls on the 16-byte chunks of scales (8 scales = tpc tiles) saves every
        // wave a chunk load it uses half of: where the default count does not divide that way and seven, six or five
        // waves do, take those (8B down, 112 tiles, chunks of 8: M = 16, K cut in two, four waves 14.0-14.3 us, seven
        // 13.4-13.6; M = 8 uncut, eight waves 11.1 us, seven 10.7).
        if (sch && M <= 16 && grid % groups == 0 && kt % (grid / groups) == 0 && group_size > 0) {
            const int tk = tile_k(bits);
            const int64_t tpc = group_size >= tk ? 8 * (int64_t)(group_size / tk) : 8 / (tk / group_size);
            const int64_t wg_tiles = kt / (grid / groups);
            auto aligned = [&](int w) { return wg_tiles % w == 0 && tpc > 0 && (wg_tiles / w) % tpc == 0; };
            if (!aligned(d.nw))
                for (int w : {7, 6, 5})
                    if (aligned(w)) { d.nw = w; break; }
        }
        // Team plan: a workgroup takes A = R x RS row blocks as RS teams that share the activations
        // through LDS (needs enough teams to stage a tile between them, and chunked scales).  It pays
        // when the activations outweigh the weights (M / (4 bits) >= 1.3 -- 1.0 at 3 bits --, or >= 1 on a larger problem) on
        // a problem long enough to hide the barrier per tile, from 17 rows up, or on very large problems.
        const bool plain_r4_uncut = r == 4 && grid == groups;
        const int64_t size = nb * K / cus;                // weight rows x columns per compute unit / 16
        const bool teams = (mb == 2 && size >= ((bf16 && bits == 4 && M <= 24) ? 20000 : 12000)) || (10 * M >= ((bits == 3 || (bits == 4 && bf16)) ? 40 : 52) * bits && size >= 20000) ||
                           (M > 8 && M >= 4 * bits && size >= 50000) || size >= 100000;
        if (!teams || !sch || force_r) return d;
        const int need = (steps_per_tile(bits) * mb + kXPiecesPerWave - 1) / kXPiecesPerWave;
        struct Cand { bool exact; int r; int64_t rs, sets; };
        std::vector<Cand> exact, shallow, deep;
        // R = 2 halves the operand reads from LDS per weight; the 3-bit instances for M > 16 are the
        // exception (no 16-wave build at R = 2, and R = 1 with twice the teams is faster)
        const int r_first = (bits == 3 && mb == 2) ? 1 : 2;
        for (int pass = 0; pass < 2; ++pass) {
            const int tr = pass == 0 ? r_first : 3 - r_first;
            if (sb % tr != 0) continue;
            // one set of row blocks per workgroup and at least 65 % of the compute units busy: no
            // fix-up; the fullest grid wins, then the larger A
            Cand best{true, tr, 0, 0};
            for (int64_t rs = 16; rs >= need; --rs) {
                const int64_t a = tr * rs;
                if (nb % a != 0) continue;
                const int64_t sets = nb / a;
                if (a >= 6 && sets <= cus && sets * 100 >= (int64_t)cus * 65 && sets > best.sets) best = Cand{true, tr, rs, sets};
                // one workgroup per compute unit, every set's K range cut across cus / sets of them:
                // up to four ("shallow") before deeper cuts
                (sets * 4 >= cus ? shallow : deep).push_back(Cand{false, tr, rs, sets});
            }
            if (best.sets) exact.push_back(best);
        }
        std::stable_sort(deep.begin(), deep.end(), [](const Cand& x, const Cand& y) { return x.sets > y.sets; });
        std::vector<Cand> order = exact;
        order.insert(order.end(), shallow.begin(), shallow.end());
        order.insert(order.end(), deep.begin(), deep.end());
        const int np = steps_per_tile(bits) * mb;         // activation pieces of one tile
        Decomp reserve = d;
        bool have_reserve = false;
        for (const Cand& c0 : order) {
            Cand c = c0;
            const int64_t cols = c.exact ? K : c.sets * K / cus;      // columns of K per workgroup
            if (cols < (bits == 4 ? 2048 : 1536)) continue;     // (4-bit: 1536 columns measured 30 % slower than the plain plan)
            // (a plain plan at R = 4 without a K cut is strong: a team plan with a K cut needs eight row blocks to
            // beat it, and does not beat it at all when it keeps 70 % of the compute units busy)
            if (!c.exact && plain_r4_uncut && (c.r * c.rs < 8 || groups * 100 >= (int64_t)cus * 70)) continue;
            // K cut across workgroups: twice the teams at R = 1 (one piece per wave where there are eight
            // or more pieces) beat R = 2 (measured, 5-17 %); with eight or more pieces per tile R = 1
            // runs best with four tiles in flight and one wave per team (3-bit: two tiles)
            if (!c.exact && np >= 8 && c.r == 2 && 2 * c.rs <= 16) { c.r = 1; c.rs *= 2; }
            const bool deep = c.r == 1 && np >= 8 && bits != 3;
            const int xpw = x_pieces_per_wave(bits, mb, (int)c.rs);
            // (3 bits up to sixteen rows: two waves per team also where K is cut across workgroups -- 70B down M = 12 / 16
            // 30.1 / 30.7 -> 28.7 / 29.5 us, bf16 34.0 / 34.1 -> 31.8 / 32.4; at 2 bits one wave per team is faster)
            int ks_first = deep ? 1 : (c.rs >= 8 ? ((c.exact || (bits == 3 && mb == 1)) ? 2 : 1) : 2);
            while (ks_first > 1 && c.rs * ks_first > 16) --ks_first;
            int nw = 0, stages = 2;
            for (int ks = ks_first; ks >= 1 && !nw; --ks) {          // fewer waves per team if the first choice does not fit
                const int w = (int)c.rs * ks;
                if (w < 4) break;
                for (int st = deep ? 4 : 2; st >= 2 && !nw; st -= 2) {
                    if (!matmul_instance_exists(bits, bf16, c.r, mb, st, true, 16, w > 8, xpw)) continue;
                    const int lds = bits == 2 ? matmul_lds_bytes<2>(c.r, mb, w, (int)c.rs, true, true)
                                  : bits == 3 ? matmul_lds_bytes<3>(c.r, mb, w, (int)c.rs, true, true)
                                              : matmul_lds_bytes<4>(c.r, mb, w, (int)c.rs, true, true);
                    if (lds > 160 * 1024) continue;
                    nw = w; stages = st;
                }
            }
            if (!nw) continue;
            // One set per workgroup that only gets one wave per team and fewer than eight waves (bf16 4-bit beyond
            // sixteen rows: no 128-register build for two pieces per wave): twice the teams, one piece per wave, every
            // set's K range cut in two, where that fits (70B gate+up bf16, M = 20..32: seven waves 75.7 us, fourteen 70.3)
            // (not for a caller with little scratch: every tile's partial sums go through it)
            if (!small_scratch && c.exact && nw < 8 && c.sets == cus && 2 * c.rs <= 16 && nb % (c.r * c.rs * 2) == 0 && K / 2 >= 2048 &&
                (int64_t)cus * c.rs * 2 <= kMaxGrid) {
                const int w2 = (int)c.rs * 2, xpw2 = x_pieces_per_wave(bits, mb, w2);
                const int lds2 = bits == 2 ? matmul_lds_bytes<2>(c.r, mb, w2, w2, true, true)
                               : bits == 3 ? matmul_lds_bytes<3>(c.r, mb, w2, w2, true, true)
                                           : matmul_lds_bytes<4>(c.r, mb, w2, w2, true, true);
                if (matmul_instance_exists(bits, bf16, c.r, mb, 2, true, 16, w2 > 8, xpw2) && lds2 <= 160 * 1024) {
                    Decomp t = d;
                    t.r = c.r; t.grid = cus; t.nw = w2; t.rs = w2; t.stages = 2;
                    return t;
                }
            }
            if ((c.exact ? c.sets : (int64_t)cus) * c.rs > kMaxGrid) continue;     // partial-sum slots of the workspace
            Decomp t = d;
            t.r = c.r; t.grid = c.exact ? (int)c.sets : cus; t.nw = nw; t.rs = (int)c.rs; t.stages = stages;
            // a 4-bit candidate that wants four tiles in flight but has no such instance (bf16 beyond eight waves) is
            // kept in reserve: a later one that has it is faster (70B QKV bf16 M = 28: ten teams, two tiles
            // 26.4 us; eight teams, four tiles 24.0 us)
            if (deep && stages == 2 && bits == 4) {
                if (!have_reserve) { reserve = t; have_reserve = true; }
                continue;
            }
            return t;
        }
        return have_reserve ? reserve : d;
    }
    if (qn == 1 && pn <= 64 && (!force_r || pn % force_r == 0)) {
        int64_t per = pn;                                 // row blocks per compute unit
        int grid = cus;
        int r = force_r ? force_r : sb;
        while (!force_r && r > 1 && per % r != 0) r >>= 1;
        if (!force_r) while (r > 2) r >>= 1;              // R <= 2 keeps two tiles in flight within 128 registers
        if (!force_r && r == 2 && per <= 16 && !wide_exists(bits, bf16, 2, mb, 2, xm) && wide_exists(bits, bf16, 1, mb, 2, xm))
            r = 1;                                        // more, narrower teams rather than half the waves
        // two row blocks per compute unit: two teams of six waves at R = 1 beat eight waves at R = 2 where
        // the work per weight is heavy (measured: bf16 4-bit 6-9 %, 2-bit at M <= 2 10-18 %); 4-bit fp16
        // and longer batches keep R = 2
        if (!force_r && r == 2 && per == 2 && wide_exists(bits, bf16, 1, mb, 2, xm) &&
            ((bits == 4 && bf16) || (bits == 2 && M <= 2) || (bits == 4 && group_size == 32 && M <= 2)))
            r = 1;                                        // (group 32, a scale per 32 weights: 8192^2 M = 1 9.6 -> 9.0-9.1 us)
        int64_t rs = per / r;
        while (rs > max_nw && rs % 2 == 0) { rs /= 2; grid *= 2; }
        const int nw = rs <= max_nw ? waves_for(r, rs, kt) : 0;
        if (nw >= 4 && nw <= max_nw && (int64_t)grid * rs <= kMaxGrid) {
            d.r = r; d.grid = grid; d.nw = nw; d.rs = (int)rs;
            return d;
        }
    } else if (!force_r && bits == 4 && qn <= 2 && pn <= 8 && bytes_per_cu >= 96 * 1024 && kt / qn >= 8) {
        const int nw = waves_for(1, pn, kt / qn);
        if (nw >= 4 && nw <= max_nw && nw % pn == 0 && (int64_t)cus * pn <= kMaxGrid) {
            d.r = 1; d.grid = cus; d.nw = nw; d.rs = (int)pn;
            return d;
        }
    }
    if (!force_r && (bits == 4 || (bits == 2 && !bf16)) && nb > 2 * (int64_t)cus) {
        // 4-bit and fp16 2-bit, row blocks that do not divide over the compute units: measured on shapes outside the
        // LLaMA-3 set (N/16 = 1376, 1728, 2000, 3696), one workgroup per compute unit or fewer, all
        // resident at once, beats several smaller ones per compute unit by 20-40 % even at 70 % of the
        // compute units busy.  A = the smallest divisor of N/16 that leaves at most one workgroup per
        // compute unit, as R = 2 x A/2 teams or A teams of R = 1.
        for (int64_t a = (nb + cus - 1) / cus; a <= 32; ++a) {
            if (nb % a != 0) continue;
            int r = (a % 2 == 0 && sb % 2 == 0 && (bits == 2 || wide_exists(bits, bf16, 2, mb, 2, xm))) ? 2 : 1;
            if (a / r > max_nw) { if (r == 1) break; continue; }
            const int64_t rs = a / r;
            const int nw = waves_for(r, rs, kt);
            if (nw >= 4 && nw <= max_nw && (nb / a) * rs <= kMaxGrid) {
                d.r = r; d.grid = (int)(nb / a); d.nw = nw; d.rs = (int)rs;
                return d;
            }
            break;
        }
    }
    if (!force_r && (bits == 4 || (bits == 2 && !bf16)) && nb > cus && nb * 2 < (int64_t)cus * 3 && sb % 2 == 0) {
        // between one and one and a half row blocks per compute unit (4-bit and fp16 2-bit): pairs of row blocks,
        // so that every workgroup is resident from the start, as R = 2 or as two teams (5120-row matrices
        // on 256 compute units, M = 4: 5120x13824 4-bit 15.1 -> 13.2 us, 2-bit 11.5 -> 9.8 us; M = 1, 2: 3-7 %)
        // (a short K as two teams of six waves, a long one as R = 2 on eight waves: 5120x5120 M = 2 7.4 us
        // at R = 2, 6.3 us as two teams; 5120x13824 is fastest at R = 2)
        const int r = (K >= 8192 && (bits == 2 || wide_exists(bits, bf16, 2, mb, 2, xm))) ? 2 : 1;
        const int64_t rs = 2 / r;
        const int nw = waves_for(r, rs, kt);
        if (nw >= 4 && nw <= max_nw) {
            d.r = r; d.grid = (int)(nb / 2); d.nw = nw; d.rs = (int)rs;
            return d;
        }
    }
    // (2- and 3-bit: measured, many small workgroups -- several per compute unit, out of step with
    // each other -- beat both a larger R and the split above: 70B QKV 3-bit 10.6 us against 12.7 us,
    // LLaMA-2-13B gate+up 3-bit 15.3 us at R = 1 against 17.6 us at R = 2)
    int r = sb;                                           // R has to divide the layout's super-block
    while (r > 1 && (bits != 4 || nb / r < cus)) r >>= 1;
    if (force_r) r = force_r;
    const int64_t groups = nb / r;
    int64_t grid = groups;
    // K is cut across workgroups only when a row group is long enough to repay the fix-up (three
    // device-scope round trips, about 2.5 us): N = 1024, K = 4096 runs in 4.3 us on 64 workgroups
    // against 6.8 us on 256
    if (groups < cus && (int64_t)r * 16 * K * bits / 8 >= 96 * 1024) {
        int64_t j = (cus + groups - 1) / groups;         // K parts per row group
        if (j > kt / 4) j = kt / 4;                      // keep at least one K tile per wavefront
        if (j < 1) j = 1;
        grid = groups * j;
    }
    // ... but two or four of them side by side as teams of one workgroup, as long as that leaves 1.6
    // workgroups per compute unit (measured at M = 1, 2, 3 on N/16 = 960 ... 3696: 32000x4096 bf16 2-bit
    // 18.4 -> 14.3 us at M = 1, 3-bit 15.5 -> 13.8 us at M = 3)
    int rs = 1;
    if (!force_r && r == 1 && grid == groups && nb <= kMaxGrid &&            // (a partial-sum slot per team and workgroup)
        (bits == 3 || (bits == 2 && bf16))) {
        for (int t : {4, 2})
            if (nb % t == 0 && nb / t >= (int64_t)cus * 16 / 10) { rs = t; break; }
        grid = groups / rs;
    }
    while (grid > kMaxGrid) grid = (grid + 1) / 2;
    d.r = r; d.grid = (int)grid; d.rs = rs;
    d.nw = (bits == 3 && grid * rs > cus) ? 4 : 8;
    return d;
}

typedef hipError_t (*matmul_launcher)(int, int, int, int, bool, int, bool, int, const MatmulParams&, hipStream_t);
typedef hipError_t (*dequant_launcher)(int, const DequantParams&, int, int, hipStream_t);

matmul_launcher pick_matmul(int bits, lutq_dtype dt) {
    if (dt == LUTQ_F16) return bits == 2 ? launch_matmul_b2_F16 : bits == 3 ? launch_matmul_b3_F16 : launch_matmul_b4_F16;
    return bits == 2 ? launch_matmul_b2_BF16 : bits == 3 ? launch_matmul_b3_BF16 : launch_matmul_b4_BF16;
}
typedef hipError_t (*rowlut_launcher)(int, int, bool, int, const MatmulParams&, hipStream_t);
rowlut_launcher pick_rowlut(int bits, lutq_dtype dt) {
    if (dt == LUTQ_F16) return bits == 2 ? launch_matmul_rowlut_b2_F16 : bits == 3 ? launch_matmul_rowlut_b3_F16 : launch_matmul_rowlut_b4_F16;
    return bits == 2 ? launch_matmul_rowlut_b2_BF16 : bits == 3 ? launch_matmul_rowlut_b3_BF16 : launch_matmul_rowlut_b4_BF16;
}
typedef hipError_t (*decode_launcher)(int, int, bool, const DecodeParams&, int, hipStream_t);
decode_launcher pick_decode(int bits, lutq_dtype dt) {
    if (dt == LUTQ_F16) return bits == 2 ? launch_decode_b2_F16 : bits == 3 ? launch_decode_b3_F16 : launch_decode_b4_F16;
    return bits == 2 ? launch_decode_b2_BF16 : bits == 3 ? launch_decode_b3_BF16 : launch_decode_b4_BF16;
}
typedef hipError_t (*rows_launcher)(int, int, int, bool, const RowsParams&, int, hipStream_t);
rows_launcher pick_rows(int bits, lutq_dtype dt) {
    if (dt == LUTQ_F16) return bits == 2 ? launch_rows_b2_F16 : bits == 3 ? launch_rows_b3_F16 : launch_rows_b4_F16;
    return bits == 2 ? launch_rows_b2_BF16 : bits == 3 ? launch_rows_b3_BF16 : launch_rows_b4_BF16;
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
        case LUTQ_ERR_GROUP: return "group_size must be 32, 64, 128 or 256 and divide K";
        case LUTQ_ERR_SHAPE: return "unsupported shape (1 <= M <= 128, N % 16 == 0, K % K-tile == 0)";
        case LUTQ_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case LUTQ_ERR_INDEX_RANGE: return "index out of range for the bit width";
        case LUTQ_ERR_WORKSPACE: return "workspace missing or too small";
        case LUTQ_ERR_DTYPE: return "dtype must be LUTQ_F16 or LUTQ_BF16";
        case LUTQ_ERR_DEVICE: return "HIP runtime error";
        case LUTQ_ERR_PLAN: return "invalid plan";
        case LUTQ_ERR_SCRATCH: return "the work decomposition needs more partial-sum scratch than lutq_matmul_static's built-in LUTQ_STATIC_SCRATCH_BYTES";
    }
    return "unknown status";
}

extern "C" size_t lutq_workspace_bytes(int64_t N, int64_t K, int bits, int group_size) {
    if (check_problem(bits, group_size, N, K) != LUTQ_OK) return 0;
    return kWorkspaceBytes;
}

extern "C" lutq_status lutq_plan_default_for(int bits, int group_size, int64_t M, int64_t N, int64_t K,
                                             lutq_dtype dtype, int compute_units, lutq_plan* plan) {
    if (!plan) return LUTQ_ERR_NULL;
    lutq_status st = check_problem(bits, group_size, N, K);
    if (st != LUTQ_OK) return st;
    if (M < 1 || M > kMaxRows || compute_units < 1 || compute_units > 4096) return LUTQ_ERR_SHAPE;
    if (dtype != LUTQ_F16 && dtype != LUTQ_BF16) return LUTQ_ERR_DTYPE;
    const bool sch = (K / group_size) % 8 == 0;
    Decomp d;
    bool wide = false;
    // beyond 32 rows: the plan of the 64-row slices where those are the default, else that of the 32-row slices
    if (M > 32 && !(wide_rows_decomp(bits, dtype == LUTQ_BF16, M < 64 ? M : 64, N, K, group_size, compute_units, &d, &wide) && wide)) {
        wide = false;
        M = 32;
    }
    if (!wide && !default_queue_decomp(bits, dtype == LUTQ_BF16, sch, M, N, K, compute_units, &d) &&
        !sliced_rows_decomp(bits, dtype == LUTQ_BF16, M, N, K, group_size, compute_units, &d) &&
        !default_rows_decomp(bits, dtype == LUTQ_BF16, M, N, K, group_size, compute_units, &d))
        d = default_decomp(bits, dtype == LUTQ_BF16, sch, M, N, K, compute_units, 0, group_size);
    plan->row_blocks_per_wave = d.r;
    plan->grid = d.grid;
    plan->waves_per_workgroup = d.nw;
    plan->tiles_in_flight = d.stages;
    plan->row_groups_per_workgroup = d.rs;
    plan->scheduling = d.rows ? LUTQ_SCHED_ROWS : d.queue ? LUTQ_SCHED_QUEUE : LUTQ_SCHED_TEAMS;
    plan->tiles_per_item = d.it;
    return LUTQ_OK;
}

extern "C" lutq_status lutq_plan_default(int bits, int group_size, int64_t M, int64_t N, int64_t K,
                                         lutq_dtype dtype, lutq_plan* plan) {
    if (!plan) return LUTQ_ERR_NULL;
    lutq_status st = check_problem(bits, group_size, N, K);
    if (st != LUTQ_OK) return st;
    if (M < 1 || M > kMaxRows) return LUTQ_ERR_SHAPE;
    if (dtype != LUTQ_F16 && dtype != LUTQ_BF16) return LUTQ_ERR_DTYPE;
    DeviceInfo di = device_info();
    if (!di.ok) return LUTQ_ERR_DEVICE;
    return lutq_plan_default_for(bits, group_size, M, N, K, dtype, di.cus, plan);
}

namespace {

// Plans registered with lutq_plan_table_set.
std::mutex g_plan_table_mu;
std::vector<lutq_plan_entry> g_plan_table;

bool plan_table_find(int bits, int group_size, int64_t M, int64_t N, int64_t K, lutq_dtype dtype, lutq_plan* out) {
    std::lock_guard<std::mutex> lock(g_plan_table_mu);
    for (const lutq_plan_entry& e : g_plan_table)
        if (e.bits == bits && e.group_size == group_size && e.dtype == dtype && e.N == N && e.K == K && e.m_min <= M && M <= e.m_max) {
            *out = e.plan;
            return true;
        }
    return false;
}

}  // namespace

extern "C" lutq_status lutq_plan_table_set(const lutq_plan_entry* entries, int count) {
    if (count < 0 || count > 4096) return LUTQ_ERR_SHAPE;
    if (count > 0 && !entries) return LUTQ_ERR_NULL;
    std::vector<lutq_plan_entry> fresh(entries, entries + count);
    std::lock_guard<std::mutex> lock(g_plan_table_mu);
    g_plan_table.swap(fresh);
    return LUTQ_OK;
}

extern "C" lutq_status lutq_plan_table_lookup(int bits, int group_size, int64_t M, int64_t N, int64_t K, lutq_dtype dtype,
                                              lutq_plan* plan) {
    if (!plan) return LUTQ_ERR_NULL;
    return plan_table_find(bits, group_size, M, N, K, dtype, plan) ? LUTQ_OK : LUTQ_ERR_PLAN;
}

namespace {

// One validated launch: everything lutq_matmul_plan decides before it touches the device.
struct Prepared {
    MatmulParams p;
    int mb, r, stages, xm;
    bool sch, wide;
    int xsh;                  // 0, or activation pieces staged per wave (shared through LDS)
    bool rowlut;              // p.lut holds one table per output row
    bool queue;               // work-queue kernel: dp and queue_lds instead of p
    bool queue_rowlut;        // ... with one table per output row
    DecodeParams dp;
    int queue_lds;
    bool rows;                // row-streaming kernel: rp, rows_lds, r = row blocks side by side
    bool rows_rowlut;         // ... with one table per output row
    RowsParams rp;
    int rows_lds;
    XopParams xp;             // ... beyond 32 rows: the operand-order copy of X made first (xp.Xop != nullptr)
};

// Validates a row-streaming launch and fills out->rp.  `d`: r = row blocks side by side (4 or 8), grid,
// nw, rs = row blocks per workgroup (the whole part of row blocks / (grid / K slices)), ks = K slices.
// `scratch`: the partial-sum area of the workspace (behind the counters): K-sliced launches keep their slots there,
// launches beyond 32 rows the operand-order copy of the activations.
lutq_status prepare_rows(const void* X, const void* packed, const void* scales, const void* lut, int bits,
                         int group_size, int64_t M, int64_t N, int64_t K, bool bf16, void* Y, const Decomp& d, Prepared* out,
                         bool rowlut = false, void* scratch = nullptr, size_t scratch_room = 0, bool dry = false) {
    const int64_t nb = N / 16, kt = K / tile_k(bits);
    if (M < 1 || M > 64) return LUTQ_ERR_SHAPE;
    const int mb = M > 32 ? (int)((M + 15) / 16) : M > 16 ? 2 : 1;
    const int ks = d.ks > 1 ? d.ks : 1;
    // beyond 32 rows the kernel reads the activations from their operand-order copy in the scratch
    const size_t xop_bytes = mb > 2 ? (size_t)(K / 32) * mb * 1024 : 0;
    if (mb > 2 && (rowlut || (!dry && (!scratch || xop_bytes > scratch_room)))) return LUTQ_ERR_PLAN;
    const int max_waves = rows_instance_waves(bits, bf16, mb, d.r);
    if (max_waves == 0 || d.nw < 4 || d.nw > max_waves || d.stages != 2) return LUTQ_ERR_PLAN;
    // K slices: grid = shares x ks workgroups; a share's row blocks in one pass; partial sums and counters in the scratch
    if (d.grid < 1 || d.grid > kMaxGrid || d.grid % ks != 0) return LUTQ_ERR_PLAN;
    const int shares = d.grid / ks;
    if (shares > nb || d.rs < 1 || d.rs > 64 || d.rs != nb / shares) return LUTQ_ERR_PLAN;
    const int extra = (int)(nb - (int64_t)d.rs * shares);
    const int amax = d.rs + (extra ? 1 : 0);
    if (ks > 1) {
        if (rowlut || mb > 2 || ks > kt || amax > d.r || (int64_t)shares * 64 > (int64_t)kCounterBytes) return LUTQ_ERR_PLAN;
        if (!dry && (!scratch || (size_t)d.grid * d.r * mb * 1024 > scratch_room)) return scratch ? LUTQ_ERR_SCRATCH : LUTQ_ERR_PLAN;
    }
    const int64_t ts = kt / ks;                               // K tiles per slice (the first kt % ks slices: one more)
    // the scales of a pass's row blocks are staged in LDS in 16-byte units: row by row with 16 bytes of padding, or, where a
    // row is not a whole number of units, as one range (shared tables only)
    const int sg2 = (int)(K / group_size) * 2;
    const bool linear = sg2 % 16 != 0;
    if (linear && rowlut) return LUTQ_ERR_PLAN;
    const int srow = linear ? sg2 : sg2 + 16;
    if (rowlut && d.r != 4) return LUTQ_ERR_PLAN;           // per-row tables: four row blocks side by side
    const int tab16 = rowlut ? rowlut16_table_bytes(bits, bf16) : 0;
    const int red_off = rows_red_off(bits, d.r, sg2, tab16);
    // rounds of the final reduction: as many row blocks at a time as LDS holds beside the table and the scales
    int rpr = rows_blocks_per_round(bits, d.r, sg2, mb, d.nw, tab16);
    if (rpr > d.r) rpr = d.r;
    if (rpr > amax) rpr = amax;
    if (rpr < 1) return LUTQ_ERR_PLAN;
    const int lds = red_off + rpr * mb * d.nw * 1024;
    RowsParams q{};
    q.X = static_cast<const uint16_t*>(X);
    q.packed = static_cast<const uint8_t*>(packed);
    q.scales = static_cast<const uint16_t*>(scales);
    q.lut = static_cast<const uint16_t*>(lut);
    q.Y = static_cast<uint16_t*>(Y);
    q.packed_bytes = (uint32_t)(N * K * bits / 8);
    q.scale_bytes = (uint32_t)(N * (K / group_size) * 2);
    q.x_bytes = (uint32_t)(M * K * 2);
    out->xp = XopParams{};
    if (mb > 2) {
        out->xp = XopParams{static_cast<const uint16_t*>(X), static_cast<uint16_t*>(scratch), (int)M, (int)K, mb, tile_k(bits) / 32};
        q.X = static_cast<const uint16_t*>(scratch);
        q.x_bytes = (uint32_t)xop_bytes;
    }
    q.M = (int)M; q.N = (int)N; q.K = (int)K; q.KT = (int)kt;
    q.SG2 = (int)(K / group_size) * 2;
    q.SBL = ilog2(super_block(nb));
    const uint32_t tile_bytes = bits == 3 ? 1536u : 1024u;
    q.tile_stride = tile_bytes << q.SBL;
    q.sblock_bytes = (uint32_t)kt * q.tile_stride;
    q.A = d.rs; q.extra = extra; q.NW = d.nw; q.G = d.grid;
    q.TQ = (int)(ts / d.nw); q.TR = (int)(ts % d.nw);
    q.KS = ks; q.TS = (int)ts; q.KSB = (int)(kt % ks);
    q.TQ1 = (int)((ts + 1) / d.nw); q.TR1 = (int)((ts + 1) % d.nw);
    q.slots = ks > 1 ? static_cast<float*>(scratch) : nullptr;
    q.counters = ks > 1 && scratch ? reinterpret_cast<uint32_t*>(static_cast<char*>(scratch) - kCounterBytes) : nullptr;   // the scratch begins with the counters
    q.RPR = rpr;
    q.s_units = linear ? 0 : sg2 / 16;
    q.s_magic = linear ? 0u : (uint32_t)((1ull << 32) / (uint64_t)q.s_units + 1);
    q.SROW = srow;
    q.red_off = red_off;
    q.tab_total = d.r * tab16;
    q.lut_ltpe = bits == 2 ? lut_log2_threads_per_row<2>(d.nw * 64)
               : bits == 3 ? lut_log2_threads_per_row<3>(d.nw * 64) : lut_log2_threads_per_row<4>(d.nw * 64);
    if (env_switches().verbose)
        std::fprintf(stderr, "lutq_matmul: row streaming, %d row blocks side by side, grid=%d (%d K slices) waves=%d row blocks per workgroup=%d (+1 in %d) reduce %d per round lds=%d\n",
                     d.r, d.grid, ks, d.nw, d.rs, extra, rpr, lds);
    out->queue = false;
    out->rows = true;
    out->rows_rowlut = rowlut;
    out->rp = q;
    out->rows_lds = lds;
    out->r = d.r;
    out->mb = mb;
    return LUTQ_OK;
}

// Validates a work-queue launch (M <= 4) and fills out->dp.  `d` holds the decomposition: r, rs = row
// groups per workgroup, nw, stages, it.
lutq_status prepare_queue(const void* X, const void* packed, const void* scales, const void* lut, int bits,
                          int group_size, int64_t M, int64_t N, int64_t K, bool bf16, void* Y, const Decomp& d, Prepared* out,
                          bool rowlut = false) {
    const int64_t nb = N / 16, kt = K / tile_k(bits);
    if (M > 4 || (K / group_size) % 8 != 0) return LUTQ_ERR_PLAN;
    if (!decode_instance_exists(bits, bf16, d.r) || super_block(nb) % d.r != 0 || (rowlut && d.r != 1)) return LUTQ_ERR_PLAN;
    const int64_t nrg = nb / d.r;
    // the row groups are dealt to the workgroups as evenly as whole row groups allow: rs each, one more
    // in the first nrg - rs * grid workgroups
    if (d.grid < 1 || d.grid > kMaxGrid || d.rs < 1 || d.rs > 64 || d.rs != nrg / d.grid) return LUTQ_ERR_PLAN;
    const int extra = (int)(nrg - (int64_t)d.rs * d.grid);
    if (d.nw < 4 || d.nw > 16 || d.stages != 2) return LUTQ_ERR_PLAN;
    if (d.it < d.stages || d.it % d.stages != 0 || kt % d.it != 0) return LUTQ_ERR_PLAN;
    const int amax = d.rs + (extra ? 1 : 0);
    const int64_t items = (int64_t)amax * (kt / d.it);
    if (items > 4096) return LUTQ_ERR_PLAN;
    if (rowlut && amax * (rowlut16_stage(bits) / 4) > 2 * d.nw * 64) return LUTQ_ERR_PLAN;   // raw tables: two words per thread
    const int lds = rowlut ? rowlut_queue_lds(bits, bf16, amax, d.nw, (int)items) : queue_lds_bytes(bits, d.nw, (int)items, d.r);
    if (lds > 160 * 1024) return LUTQ_ERR_PLAN;
    DecodeParams q{};
    q.X = static_cast<const uint16_t*>(X);
    q.packed = static_cast<const uint8_t*>(packed);
    q.scales = static_cast<const uint16_t*>(scales);
    q.lut = static_cast<const uint16_t*>(lut);
    q.Y = static_cast<uint16_t*>(Y);
    q.packed_bytes = (uint32_t)(N * K * bits / 8);
    q.scale_bytes = (uint32_t)(N * (K / group_size) * 2);
    q.x_bytes = (uint32_t)(M * K * 2);
    q.M = (int)M; q.N = (int)N; q.K = (int)K;
    q.SG2 = (int)(K / group_size) * 2;
    q.SBL = ilog2(super_block(nb));
    const uint32_t tile_bytes = bits == 3 ? 1536u : 1024u;
    q.tile_stride = tile_bytes << q.SBL;
    q.sblock_bytes = (uint32_t)kt * q.tile_stride;
    q.A = d.rs; q.extra = extra; q.C = (int)(kt / d.it); q.IT = d.it; q.NW = d.nw; q.G = d.grid;
    q.a_magic = q.A == 1 ? 0xffffffffu : (uint32_t)((1ull << 32) / (uint64_t)q.A);
    q.a1_magic = (uint32_t)((1ull << 32) / (uint64_t)(q.A + 1));
    // the waves that build the shared table: the first eight of sixteen (about 1 % on 70B gate+up and down: 41.7 -> 41.2
    // and 22.1 -> 21.8 us in one A/B, within the noise in another); with twelve waves all of them (eight builders and
    // four late waves measured 2-3 % slower on 8B gate+up and 70B QKV)
    q.NB = d.nw < 16 || rowlut ? d.nw : 8;
    q.lut_ltpe = bits == 2 ? lut_log2_threads_per_row<2>(q.NB * 64)
               : bits == 3 ? lut_log2_threads_per_row<3>(q.NB * 64) : lut_log2_threads_per_row<4>(q.NB * 64);
    q.slot_off = bits == 2 ? decode_slot_off<2>(d.nw) : bits == 3 ? decode_slot_off<3>(d.nw) : decode_slot_off<4>(d.nw);
    q.tab_total = 0;
    if (rowlut) {
        q.tab_total = amax * rowlut16_table_bytes(bits, bf16);
        q.slot_off = q.tab_total + 256 + d.nw * 1024;
    }
    // final reduction: as many groups of items per output as there are threads for them (the group sums
    // are parked in the table's area: at most 4 KiB)
    const int outputs = q.A * d.r * 64, outputs_max = amax * d.r * 64;
    int ng = (d.nw * 64) / outputs_max;
    if (ng > q.C / 8) ng = q.C / 8;                       // groups of eight items or more: fewer are not worth a barrier
    if (ng < 1) ng = 1;
    q.GL = (q.C + ng - 1) / ng;
    q.NG = (q.C + q.GL - 1) / q.GL;
    q.o_magic = (uint32_t)((1ull << 32) / (uint64_t)outputs);
    q.o1_magic = (uint32_t)((1ull << 32) / (uint64_t)(outputs + d.r * 64));
    q.trace = nullptr;
    if (env_switches().verbose)
        std::fprintf(stderr, "lutq_matmul: work queue R=%d grid=%d waves=%d row groups per workgroup=%d tiles per item=%d items=%d lds=%d\n",
                     d.r, d.grid, d.nw, d.rs, d.it, (int)items, lds);
    out->queue = true;
    out->queue_rowlut = rowlut;
    out->dp = q;
    out->queue_lds = lds;
    out->r = d.r;
    return LUTQ_OK;
}

// Validates the arguments of one launch (M <= 32) and fills *out; launches nothing.
lutq_status prepare_matmul(const void* X, const void* packed, const void* scales, const void* lut,
                           int bits, int group_size, int64_t M, int64_t N, int64_t K,
                           lutq_dtype dtype, void* Y, void* workspace, size_t workspace_bytes,
                           const lutq_plan* user_plan, bool rowlut, int dry_run_cus, Prepared* out,
                           bool fitted_workspace = false, bool consult_table = true, bool small_scratch = false) {
    // no plan from the caller: a registered plan for this call goes first, if the kernels can run it
    lutq_plan registered;
    if (!user_plan && !rowlut && dry_run_cus == 0 && consult_table &&
        plan_table_find(bits, group_size, M, N, K, dtype, &registered)) {
        const lutq_status st = prepare_matmul(X, packed, scales, lut, bits, group_size, M, N, K, dtype, Y, workspace,
                                              workspace_bytes, &registered, rowlut, dry_run_cus, out, fitted_workspace, false);
        if (st != LUTQ_ERR_PLAN && st != LUTQ_ERR_SCRATCH) return st;
    }
    // dry_run_cus > 0: only the plan is checked, for a device of that many compute units; no pointer is
    // looked at and no device is queried
    const bool dry = dry_run_cus > 0;
    if (!dry && (!X || !packed || !scales || !lut || !Y)) return LUTQ_ERR_NULL;
    lutq_status st = check_problem(bits, group_size, N, K);
    if (st != LUTQ_OK) return st;
    if (M < 1 || M > 32) return LUTQ_ERR_SHAPE;
    if (dtype != LUTQ_F16 && dtype != LUTQ_BF16) return LUTQ_ERR_DTYPE;
    DeviceInfo di;
    if (dry) {
        di.cus = dry_run_cus; di.ok = true;
    } else {
        if (!aligned16(X) || !aligned16(packed) || !aligned16(scales) || !aligned16(Y) || !aligned16(workspace))
            return LUTQ_ERR_ALIGN;
        if ((reinterpret_cast<uintptr_t>(lut) & 1u) != 0 || (rowlut && !aligned16(lut))) return LUTQ_ERR_ALIGN;
        // fitted_workspace: the scratch is checked further down against what this launch really uses
        if (!workspace || workspace_bytes < (fitted_workspace ? kCounterBytes : kWorkspaceBytes)) return LUTQ_ERR_WORKSPACE;
        di = device_info();
        if (!di.ok) {
            if (env_switches().verbose) std::fprintf(stderr, "lutq_matmul: device query failed: %s\n", hipGetErrorString(hipGetLastError()));
            return LUTQ_ERR_DEVICE;
        }
    }
    const int64_t nb = N / 16, kt = K / tile_k(bits);
    const int mb = M > 16 ? 2 : 1;
    const bool bf16 = dtype == LUTQ_BF16;
    // M <= 4: four K steps of activations per load, rotated into place (a quarter of the registers);
    // M <= 8: two, unless the plan shares the activations through LDS (decided below)
    int xm = (M <= 4) ? 4 : 16;
    const bool sch = (K / group_size) % 8 == 0;            // scale rows are 16-byte aligned: chunked scale path
    int force_r = 0;
    if (user_plan) {
        const int w = user_plan->waves_per_workgroup, f = user_plan->tiles_in_flight;
        const int t = user_plan->row_groups_per_workgroup;
        const bool teams = user_plan->scheduling == 0 || user_plan->scheduling == LUTQ_SCHED_TEAMS;
        if ((w != 0 && (w < 4 || w > 16)) || (f != 0 && f != 2 && f != 4) || t < 0 || t > (teams ? 16 : 64)) return LUTQ_ERR_PLAN;
        force_r = user_plan->row_blocks_per_wave;
        if (teams && force_r != 0 && ((force_r != 1 && force_r != 2 && force_r != 4) || super_block(nb) % force_r != 0))
            return LUTQ_ERR_PLAN;
        if (user_plan->grid != 0 && (user_plan->grid < 1 || user_plan->grid > kMaxGrid)) return LUTQ_ERR_PLAN;
    }
    out->queue = false;
    out->queue_rowlut = false;
    out->rows = false;
    out->rows_rowlut = false;
    if (rowlut && user_plan && user_plan->scheduling > LUTQ_SCHED_TEAMS) return LUTQ_ERR_PLAN;
    if (rowlut && !user_plan && M > 4 && nb >= 2 * (int64_t)di.cus && ((K / group_size) * 2) % 16 == 0) {
        // one table per output row, 5..32 rows, at least two row blocks per compute unit: the row-streaming
        // kernel with the tables of four row blocks at a time (the teams' per-row-table kernel holds one row
        // block's and fetches the activations again for every row block)
        const int grid = di.cus;
        const int64_t per = nb / grid;
        int nw = rows_instance_waves(bits, bf16, mb, 4);
        if (nw > kt) nw = (int)(kt < 4 ? 4 : kt);
        if (per <= 64 && nw >= 4 && rows_blocks_per_round(bits, 4, (int)(K / group_size) * 2, mb, nw, rowlut16_table_bytes(bits, bf16)) >= 1) {
            Decomp q;
            q.r = 4; q.grid = grid; q.nw = nw; q.stages = 2; q.rs = (int)per; q.queue = 0; q.it = 0; q.rows = 1;
            const lutq_status qs = prepare_rows(X, packed, scales, lut, bits, group_size, M, N, K, bf16, Y, q, out, true);
            if (qs == LUTQ_OK) return qs;
            out->rows = false;
            out->rows_rowlut = false;
        }
    }
    if (rowlut && !user_plan) {
        // one table per output row, M <= 4: the work-queue kernel with all of a workgroup's tables resident
        Decomp q;
        if (rowlut_queue_decomp(bits, bf16, sch, M, N, K, di.cus, &q)) {
            const lutq_status qs = prepare_queue(X, packed, scales, lut, bits, group_size, M, N, K, bf16, Y, q, out, true);
            if (qs == LUTQ_OK) return qs;
            out->queue = false;
            out->queue_rowlut = false;
        }
    }
    if (!rowlut) {
        // the work-queue kernel: asked for by the plan, or the default for M <= 4 where it applies
        // (an explicit plan without a scheduling field keeps meaning the static teams it describes)
        const bool plan_is_empty = !user_plan || (user_plan->row_blocks_per_wave == 0 && user_plan->grid == 0 &&
                                                  user_plan->waves_per_workgroup == 0 && user_plan->tiles_in_flight == 0 &&
                                                  user_plan->row_groups_per_workgroup == 0 && user_plan->tiles_per_item == 0);
        const int sched = user_plan ? user_plan->scheduling : 0;
        if (sched < 0 || sched > LUTQ_SCHED_ROWS) return LUTQ_ERR_PLAN;
        Decomp q;
        if (sched == LUTQ_SCHED_ROWS) {
            // tiles_per_item: K tiles per slice where K is cut across workgroups (grid = shares x slices)
            int ks = 1;
            if (user_plan->tiles_per_item != 0) {
                if (user_plan->tiles_per_item < 1 || !user_plan->grid) return LUTQ_ERR_PLAN;
                ks = (int)((kt + user_plan->tiles_per_item - 1) / user_plan->tiles_per_item);    // slices as even as whole tiles allow
                if (ks < 2 || user_plan->grid % ks != 0) return LUTQ_ERR_PLAN;
            }
            const bool have_default = rows_decomp(bits, bf16, M, N, K, group_size, di.cus, &q);
            if (!have_default) { q.r = 4; q.grid = (int)(nb < di.cus ? nb : di.cus); q.nw = 8; q.stages = 2; }
            if (user_plan->row_blocks_per_wave) {
                q.r = user_plan->row_blocks_per_wave;
                const int w = rows_instance_waves(bits, bf16, mb, q.r);
                if (!user_plan->waves_per_workgroup && w) q.nw = (int)(w > kt ? (kt < 4 ? 4 : kt) : w);
            }
            if (user_plan->grid) q.grid = user_plan->grid;
            else if (user_plan->row_groups_per_workgroup) {
                if (nb % user_plan->row_groups_per_workgroup != 0) return LUTQ_ERR_PLAN;
                q.grid = (int)(nb / user_plan->row_groups_per_workgroup);
            }
            if (q.grid < 1 || q.grid / ks > nb) return LUTQ_ERR_PLAN;
            q.rs = (int)(nb / (q.grid / ks));
            q.ks = ks;
            q.it = ks > 1 ? user_plan->tiles_per_item : 0;
            if (user_plan->row_groups_per_workgroup && user_plan->row_groups_per_workgroup != q.rs) return LUTQ_ERR_PLAN;
            if (user_plan->waves_per_workgroup) q.nw = user_plan->waves_per_workgroup;
            if (user_plan->tiles_in_flight) q.stages = user_plan->tiles_in_flight;
            if (ks > 1) {
                const lutq_status rs = prepare_rows(X, packed, scales, lut, bits, group_size, M, N, K, bf16, Y, q, out, false,
                                                    dry ? nullptr : static_cast<char*>(workspace) + kCounterBytes,
                                                    dry ? 0 : workspace_bytes - kCounterBytes, dry);
                return rs;
            }
            return prepare_rows(X, packed, scales, lut, bits, group_size, M, N, K, bf16, Y, q, out);
        }
        if (sched == LUTQ_SCHED_QUEUE) {
            // the fields the plan leaves open: one workgroup per compute unit where the row blocks divide
            // evenly, else one workgroup of 16 waves per row block with items of two tiles
            const bool have_default = queue_decomp(bits, bf16, sch, M, N, K, di.cus, false, &q);
            if (!have_default) {
                q.r = 1; q.rs = 1; q.nw = 16; q.stages = 2; q.it = 2; q.queue = 1;
            }
            if (user_plan->row_blocks_per_wave) q.r = user_plan->row_blocks_per_wave;
            if (q.r != 1 && q.r != 2) return LUTQ_ERR_PLAN;
            if (nb % q.r != 0) return LUTQ_ERR_PLAN;
            const int64_t nrg = nb / q.r;
            // grid and row groups per workgroup: either fixes the other (row groups per workgroup = the
            // whole part of row groups / grid; a grid derived from them has to come out even)
            if (user_plan->grid) {
                q.grid = user_plan->grid;
                q.rs = (int)(nrg / q.grid);
                if (user_plan->row_groups_per_workgroup && user_plan->row_groups_per_workgroup != q.rs) return LUTQ_ERR_PLAN;
            } else {
                if (user_plan->row_groups_per_workgroup) q.rs = user_plan->row_groups_per_workgroup;
                else if (user_plan->row_blocks_per_wave && have_default) q.rs = (int)(nrg / di.cus);
                if (q.rs < 1 || nrg % q.rs != 0) return LUTQ_ERR_PLAN;
                q.grid = (int)(nrg / q.rs);
            }
            if (user_plan->waves_per_workgroup) q.nw = user_plan->waves_per_workgroup;
            if (user_plan->tiles_in_flight) q.stages = user_plan->tiles_in_flight;
            if (user_plan->tiles_per_item) q.it = user_plan->tiles_per_item;
            return prepare_queue(X, packed, scales, lut, bits, group_size, M, N, K, bf16, Y, q, out);
        }
        if (sched == 0 && plan_is_empty && default_queue_decomp(bits, bf16, sch, M, N, K, di.cus, &q))
            return prepare_queue(X, packed, scales, lut, bits, group_size, M, N, K, bf16, Y, q, out);
        if (sched == 0 && plan_is_empty && sliced_rows_decomp(bits, bf16, M, N, K, group_size, di.cus, &q)) {
            // (a scratch too small for the slices' sums -- the built-in one of lutq_matmul_static -- leaves it to the others)
            const lutq_status rs = prepare_rows(X, packed, scales, lut, bits, group_size, M, N, K, bf16, Y, q, out, false,
                                                dry ? nullptr : static_cast<char*>(workspace) + kCounterBytes,
                                                dry ? 0 : workspace_bytes - kCounterBytes, dry);
            if (rs == LUTQ_OK) return rs;
            out->rows = false;
            q = Decomp{};
        }
        if (sched == 0 && plan_is_empty && default_rows_decomp(bits, bf16, M, N, K, group_size, di.cus, &q))
            return prepare_rows(X, packed, scales, lut, bits, group_size, M, N, K, bf16, Y, q, out);
    }
    Decomp d = default_decomp(bits, bf16, sch, M, N, K, di.cus, force_r, group_size, small_scratch);
    if (rowlut) {
        // one table per output row: a workgroup holds the tables of one row block at a time, so one
        // row block per workgroup, its K range split over eight waves, and over several workgroups
        // when there are fewer row blocks than compute units
        int64_t grid = nb;
        if (nb < (int64_t)di.cus * 6 / 10) {
            int64_t j = (di.cus + nb - 1) / nb;
            if (j > kt / 4) j = kt / 4;
            if (j < 1) j = 1;
            grid = nb * j;
        }
        if (grid > kMaxGrid) grid = kMaxGrid;
        d.r = 1; d.rs = 1; d.nw = 8; d.stages = 2; d.grid = (int)grid;
    }
    if (user_plan) {
        // a field the caller fixes replaces the default; teams and waves default to one team of the
        // default number of waves once anything about the workgroup's shape is fixed by the caller
        const bool shaped = user_plan->grid || user_plan->waves_per_workgroup || user_plan->row_groups_per_workgroup;
        if (shaped) {
            d.rs = user_plan->row_groups_per_workgroup ? user_plan->row_groups_per_workgroup : 1;
            d.nw = user_plan->waves_per_workgroup ? user_plan->waves_per_workgroup : (d.rs > 4 ? d.rs : 4);
            if (!user_plan->grid) d.grid = (int)((nb / d.r / d.rs) > 0 ? (nb / d.r / d.rs) : 1);
            if (!user_plan->tiles_in_flight) d.stages = 2;
        }
        if (user_plan->grid) d.grid = user_plan->grid;
        if (user_plan->tiles_in_flight) d.stages = user_plan->tiles_in_flight;
    }
    if (!sch) { if (d.nw > 8) d.nw = 8 / d.rs > 0 ? (8 / d.rs) * d.rs : d.rs; d.stages = 2; }   // per-tile scale path: one shape only
    const int r = d.r;
    const int64_t nrg = nb / r;
    if (d.nw % d.rs != 0 || nrg % d.rs != 0 || d.nw < 4 || d.nw > 16) return LUTQ_ERR_PLAN;
    const int64_t tiles = (nrg / d.rs) * kt;
    if (d.grid > tiles) d.grid = (int)tiles;              // every workgroup must own at least one iteration
    if ((int64_t)d.grid * d.rs > kMaxGrid) return LUTQ_ERR_PLAN;   // partial-sum slots of the workspace
    // more than 8 waves need an instance held to 128 registers; up to 8 waves take one when it
    // exists, so that two workgroups fit a compute unit
    // M > 4 with enough teams: the activations are staged in LDS once per workgroup instead of being
    // fetched by every team (LUTQ_NO_SHARED_X=1 switches that off, for comparisons)
    int xsh = (!rowlut && M > 4 && sch && teams_can_share_x(bits, mb, d.rs) && !env_switches().no_shared_x)
                  ? x_pieces_per_wave(bits, mb, d.rs) : 0;
    const bool can_pack8 = M > 4 && M <= 8 && !env_switches().no_xm8;
    if (can_pack8 && !xsh) xm = 8;
    bool wide = d.nw > 8 || (d.nw > 4 && sch && matmul_instance_exists(bits, bf16, r, mb, d.stages, sch, xm, true, xsh));
    if (xsh && !matmul_instance_exists(bits, bf16, r, mb, d.stages, sch, xm, wide, xsh)) {
        xsh = 0;
        if (can_pack8) xm = 8;
        wide = d.nw > 8 || (d.nw > 4 && sch && wide_exists(bits, bf16, r, mb, d.stages, xm));
    }
    if (!matmul_instance_exists(bits, bf16, r, mb, d.stages, sch, xm, wide, xsh)) return LUTQ_ERR_PLAN;
    int lds_bytes = bits == 2 ? matmul_lds_bytes<2>(r, mb, d.nw, d.rs, sch, xsh)
                  : bits == 3 ? matmul_lds_bytes<3>(r, mb, d.nw, d.rs, sch, xsh)
                              : matmul_lds_bytes<4>(r, mb, d.nw, d.rs, sch, xsh);
    if (xsh && lds_bytes > 160 * 1024) {                  // the buffers do not fit: fetch per team
        xsh = 0;
        if (can_pack8) xm = 8;
        wide = d.nw > 8 || (d.nw > 4 && sch && wide_exists(bits, bf16, r, mb, d.stages, xm));
        if (!matmul_instance_exists(bits, bf16, r, mb, d.stages, sch, xm, wide, false)) return LUTQ_ERR_PLAN;
        lds_bytes = bits == 2 ? matmul_lds_bytes<2>(r, mb, d.nw, d.rs, sch, false)
                  : bits == 3 ? matmul_lds_bytes<3>(r, mb, d.nw, d.rs, sch, false)
                              : matmul_lds_bytes<4>(r, mb, d.nw, d.rs, sch, false);
    }
    if (lds_bytes > 160 * 1024) return LUTQ_ERR_PLAN;
    if (fitted_workspace) {
        // partial sums leave a workgroup only if some range of iterations ends inside an output tile
        const bool splits = tiles % d.grid != 0 || (tiles / d.grid) % kt != 0;
        const size_t need = splits ? (size_t)d.grid * 2 * d.rs * slot_floats(r, mb) * sizeof(float) : 0;
        if (kCounterBytes + need > workspace_bytes) {
            // the library's own choice does not fit the caller's scratch: once more with the plans that need little
            if (!user_plan && !small_scratch)
                return prepare_matmul(X, packed, scales, lut, bits, group_size, M, N, K, dtype, Y, workspace, workspace_bytes,
                                      user_plan, rowlut, dry_run_cus, out, fitted_workspace, false, true);
            return LUTQ_ERR_SCRATCH;
        }
    }

    MatmulParams p;
    p.X = static_cast<const uint16_t*>(X);
    p.packed = static_cast<const uint8_t*>(packed);
    p.scales = static_cast<const uint16_t*>(scales);
    p.lut = static_cast<const uint16_t*>(lut);
    p.Y = static_cast<uint16_t*>(Y);
    p.counters = static_cast<uint32_t*>(workspace);
    p.slots = dry ? nullptr : reinterpret_cast<float*>(static_cast<char*>(workspace) + kCounterBytes);
    p.packed_bytes = (uint32_t)(N * K * bits / 8);
    p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.KT = (int)kt;
    p.NRG = (int)nrg;
    p.G = d.grid;
    p.TQ = (int)(tiles / d.grid);
    p.TR = (int)(tiles % d.grid);
    p.SG = (int)(K / group_size);
    p.SBL = ilog2(super_block(nb));
    p.NW = d.nw; p.RS = d.rs; p.KS = d.nw / d.rs;
    p.xbuf_off = bits == 2 ? matmul_xbuf_offset<2>(r, mb, d.nw, d.rs, sch)
               : bits == 3 ? matmul_xbuf_offset<3>(r, mb, d.nw, d.rs, sch) : matmul_xbuf_offset<4>(r, mb, d.nw, d.rs, sch);
    p.lut_ltpe = bits == 2 ? lut_log2_threads_per_row<2>(d.nw * 64)
               : bits == 3 ? lut_log2_threads_per_row<3>(d.nw * 64) : lut_log2_threads_per_row<4>(d.nw * 64);
    p.kt_magic = p.KT == 1 ? 0xffffffffu : (uint32_t)((1ull << 32) / (uint64_t)p.KT);
    p.ks_magic = p.KS == 1 ? 0xffffffffu : (uint32_t)((1ull << 32) / (uint64_t)p.KS);
    p.fast_reduce = (d.nw - d.rs) * (r * mb * 4) * 256 <= (bits == 3 ? 64 : 256) * 256 ? 1 : 0;
    p.trace = nullptr;
    if (env_switches().verbose)
        std::fprintf(stderr, "lutq_matmul: R=%d grid=%d waves=%d (teams %d x %d) stages=%d wide=%d xm=%d shared_x=%d lds=%d\n", r, d.grid,
                     d.nw, d.rs, p.KS, d.stages, (int)wide, xm, (int)xsh, lds_bytes);
    out->p = p;
    out->mb = mb; out->r = r; out->stages = d.stages; out->xm = xm;
    out->sch = sch; out->wide = wide; out->xsh = xsh; out->rowlut = rowlut;
    return LUTQ_OK;
}

lutq_status launch_prepared(const Prepared& q, int bits, int group_size, lutq_dtype dtype, void* stream) {
    if (q.rows) {
        if (q.xp.Xop) {
            hipLaunchKernelGGL(rows_xop_kernel, dim3((unsigned)q.rp.KT, (unsigned)q.xp.MB), dim3(256), 0, static_cast<hipStream_t>(stream), q.xp);
            if (hipGetLastError() != hipSuccess) return LUTQ_ERR_DEVICE;
        }
        const hipError_t e = pick_rows(bits, dtype)(group_size, q.mb, q.r, q.rows_rowlut, q.rp, q.rows_lds, static_cast<hipStream_t>(stream));
        if (e != hipSuccess && env_switches().verbose)
            std::fprintf(stderr, "lutq_matmul: launch failed: %s (grid %d, block %d, lds %d)\n", hipGetErrorString(e), q.rp.G, q.rp.NW * 64, q.rows_lds);
        return e == hipSuccess ? LUTQ_OK : LUTQ_ERR_DEVICE;
    }
    if (q.queue) {
        const hipError_t e = pick_decode(bits, dtype)(group_size, q.r, q.queue_rowlut, q.dp, q.queue_lds, static_cast<hipStream_t>(stream));
        return e == hipSuccess ? LUTQ_OK : LUTQ_ERR_DEVICE;
    }
    hipError_t e = q.rowlut ? pick_rowlut(bits, dtype)(group_size, q.mb, q.sch, q.xm, q.p, static_cast<hipStream_t>(stream))
                            : pick_matmul(bits, dtype)(group_size, q.mb, q.r, q.stages, q.sch, q.xm, q.wide, q.xsh, q.p,
                                                       static_cast<hipStream_t>(stream));
    if (e != hipSuccess && env_switches().verbose)
        std::fprintf(stderr, "lutq_matmul: launch failed: %s (grid %d, block %d)\n", hipGetErrorString(e), q.p.G, q.p.NW * 64);
    return e == hipSuccess ? LUTQ_OK : LUTQ_ERR_DEVICE;
}

}  // namespace

namespace {

// How a call's activation rows are cut into launches: slices of 64 rows through the row-streaming kernel where
// that exists and is the default (or the plan asks for it: scheduling = LUTQ_SCHED_ROWS), else slices of 32.
// Returns the slice height; *d holds the 64-row decomposition (its waves are those of a full slice).
int slice_rows(int bits, int group_size, int64_t M, int64_t N, int64_t K, bool bf16, const lutq_plan* user_plan, bool rowlut,
               int cus, lutq_status* st) {
    *st = LUTQ_OK;
    if (M <= 32 || rowlut) return 32;
    const bool plan_is_empty = !user_plan || (user_plan->row_blocks_per_wave == 0 && user_plan->grid == 0 &&
                                              user_plan->waves_per_workgroup == 0 && user_plan->tiles_in_flight == 0 &&
                                              user_plan->row_groups_per_workgroup == 0 && user_plan->tiles_per_item == 0);
    const int sched = user_plan ? user_plan->scheduling : 0;
    if (sched != LUTQ_SCHED_ROWS && !(sched == 0 && plan_is_empty)) return 32;
    // a row-streaming plan with K slices describes launches of up to 32 rows
    if (sched == LUTQ_SCHED_ROWS && user_plan->tiles_per_item != 0) return 32;
    Decomp d;
    bool take = false;
    const bool have = wide_rows_decomp(bits, bf16, M < 64 ? M : 64, N, K, group_size, cus, &d, &take);
    if (sched == LUTQ_SCHED_ROWS) {
        // beyond 32 rows the row-streaming plan has no free fields: each is zero or the one value there is
        auto fixed = [](int given, int only) { return given == 0 || given == only; };
        if (!have || !fixed(user_plan->row_blocks_per_wave, d.r) || !fixed(user_plan->grid, d.grid) ||
            !fixed(user_plan->waves_per_workgroup, d.nw) || !fixed(user_plan->tiles_in_flight, d.stages) ||
            !fixed(user_plan->row_groups_per_workgroup, d.rs) || user_plan->tiles_per_item != 0)
            *st = LUTQ_ERR_PLAN;
        return 64;
    }
    return have && take ? 64 : 32;
}

lutq_status matmul_sliced(const void* X, const void* packed, const void* scales, const void* lut,
                          int bits, int group_size, int64_t M, int64_t N, int64_t K,
                          lutq_dtype dtype, void* Y, void* workspace, size_t workspace_bytes,
                          void* stream, const lutq_plan* user_plan, bool rowlut, bool fitted_workspace = false, bool pairs = false) {
    if (!X || !Y) return LUTQ_ERR_NULL;
    // a codebook of pairs (4-bit layout) or quads (2-bit layout): one byte = one codebook index, entries read as aligned 32-bit words
    if (pairs && bits != 4 && bits != 2) return LUTQ_ERR_BITS;
    if (pairs && (reinterpret_cast<uintptr_t>(lut) & 3u) != 0) return LUTQ_ERR_ALIGN;
    if (M < 1 || M > kMaxRows) return LUTQ_ERR_SHAPE;
    // More than 32 activation rows: slices of 32 rows (64 where the row-streaming kernel takes them in one pass
    // over the weights), one launch each on the same stream (the weights are streamed once per slice).  Every
    // slice is validated before the first launch.
    int64_t step = 32;
    if (M > 32) {
        lutq_status st = check_problem(bits, group_size, N, K);
        if (st != LUTQ_OK) return st;
        if (dtype != LUTQ_F16 && dtype != LUTQ_BF16) return LUTQ_ERR_DTYPE;
        const DeviceInfo di = device_info();
        if (!di.ok) return LUTQ_ERR_DEVICE;
        step = slice_rows(bits, group_size, M, N, K, dtype == LUTQ_BF16, user_plan, rowlut, di.cus, &st);
        if (st != LUTQ_OK) return st;
    }
    const int64_t full = M / step, rest = M % step;
    Prepared body{}, tail{};
    const size_t xrow = (size_t)K * 2, yrow = (size_t)N * 2;
    // one slice of m rows (m <= step) starting at row m0
    auto prepare = [&](int64_t m0, int64_t m, Prepared* out) -> lutq_status {
        const void* Xs = static_cast<const char*>(X) + (size_t)m0 * xrow;
        void* Ys = static_cast<char*>(Y) + (size_t)m0 * yrow;
        if (m <= 32)
            return prepare_matmul(Xs, packed, scales, lut, bits, group_size, m, N, K, dtype, Ys, workspace, workspace_bytes,
                                  step == 64 ? nullptr : user_plan, rowlut, 0, out, fitted_workspace);
        if (!packed || !scales || !lut) return LUTQ_ERR_NULL;
        if (!aligned16(X) || !aligned16(packed) || !aligned16(scales) || !aligned16(Y) || !aligned16(workspace) ||
            (reinterpret_cast<uintptr_t>(lut) & 1u) != 0)
            return LUTQ_ERR_ALIGN;
        if (!workspace || workspace_bytes < (fitted_workspace ? kCounterBytes : kWorkspaceBytes)) return LUTQ_ERR_WORKSPACE;
        Decomp d;
        bool take = false;
        if (!wide_rows_decomp(bits, dtype == LUTQ_BF16, m, N, K, group_size, device_info().cus, &d, &take)) return LUTQ_ERR_PLAN;
        // the operand-order copy of the slice's activations lives where other launches keep their partial sums
        const lutq_status st = prepare_rows(Xs, packed, scales, lut, bits, group_size, m, N, K, dtype == LUTQ_BF16, Ys, d, out, false,
                                            static_cast<char*>(workspace) + kCounterBytes, workspace_bytes - kCounterBytes);
        return st == LUTQ_ERR_PLAN && fitted_workspace ? LUTQ_ERR_SCRATCH : st;
    };
    if (full > 0) {
        const lutq_status st = prepare(0, step, &body);
        if (st != LUTQ_OK) return st;
    }
    if (rest > 0) {
        const lutq_status st = prepare(full * step, rest, &tail);
        if (st != LUTQ_OK) return st;
    }
    if (pairs) {
        // the kernels' table build takes the caller's 256 pairs or quads as the vectorised table itself
        for (Prepared* q : {&body, &tail}) {
            q->p.lut_ltpe |= kLutPairsFlag;
            q->dp.lut_ltpe |= kLutPairsFlag;
            q->rp.lut_ltpe |= kLutPairsFlag;
        }
    }
    for (int64_t i = 0; i < full; ++i) {
        Prepared q = body;
        q.p.X = reinterpret_cast<const uint16_t*>(static_cast<const char*>(X) + (size_t)i * step * xrow);
        q.p.Y = reinterpret_cast<uint16_t*>(static_cast<char*>(Y) + (size_t)i * step * yrow);
        if (q.xp.Xop) q.xp.X = q.p.X;       // the kernel reads the copy, which is made from this slice's rows
        else q.rp.X = q.p.X;
        q.rp.Y = q.p.Y;
        lutq_status st = launch_prepared(q, bits, group_size, dtype, stream);
        if (st != LUTQ_OK) return st;
    }
    return rest > 0 ? launch_prepared(tail, bits, group_size, dtype, stream) : LUTQ_OK;
}

}  // namespace

extern "C" lutq_status lutq_plan_check(int bits, int group_size, int64_t M, int64_t N, int64_t K, lutq_dtype dtype,
                                       int compute_units, const lutq_plan* plan) {
    if (compute_units < 1 || compute_units > 4096 || M < 1 || M > kMaxRows) return LUTQ_ERR_SHAPE;
    Prepared q{};
    int64_t step = 32;
    if (M > 32) {
        lutq_status st = check_problem(bits, group_size, N, K);
        if (st != LUTQ_OK) return st;
        if (dtype != LUTQ_F16 && dtype != LUTQ_BF16) return LUTQ_ERR_DTYPE;
        step = slice_rows(bits, group_size, M, N, K, dtype == LUTQ_BF16, plan, false, compute_units, &st);
        if (st != LUTQ_OK) return st;
    }
    for (int64_t m : {M >= step ? step : (int64_t)0, M % step}) {      // the full slices, then the rest
        if (m == 0) continue;
        lutq_status st;
        if (m <= 32) {
            st = prepare_matmul(nullptr, nullptr, nullptr, nullptr, bits, group_size, m, N, K, dtype, nullptr,
                                nullptr, 0, step == 64 ? nullptr : plan, false, compute_units, &q);
        } else {
            Decomp d;
            bool take = false;
            if (!wide_rows_decomp(bits, dtype == LUTQ_BF16, m, N, K, group_size, compute_units, &d, &take)) return LUTQ_ERR_PLAN;
            st = prepare_rows(nullptr, nullptr, nullptr, nullptr, bits, group_size, m, N, K, dtype == LUTQ_BF16, nullptr, d, &q,
                              false, nullptr, 0, true);
        }
        if (st != LUTQ_OK) return st;
    }
    return LUTQ_OK;
}

extern "C" lutq_status lutq_matmul_plan(const void* X, const void* packed, const void* scales, const void* lut,
                                        int bits, int group_size, int64_t M, int64_t N, int64_t K,
                                        lutq_dtype dtype, void* Y, void* workspace, size_t workspace_bytes,
                                        void* stream, const lutq_plan* user_plan) {
    return matmul_sliced(X, packed, scales, lut, bits, group_size, M, N, K, dtype, Y, workspace, workspace_bytes,
                         stream, user_plan, false);
}

extern "C" lutq_status lutq_matmul_channel(const void* X, const void* packed, const void* scales, const void* luts,
                                           int bits, int group_size, int64_t M, int64_t N, int64_t K,
                                           lutq_dtype dtype, void* Y, void* workspace, size_t workspace_bytes,
                                           void* stream) {
    return matmul_sliced(X, packed, scales, luts, bits, group_size, M, N, K, dtype, Y, workspace, workspace_bytes,
                         stream, nullptr, true);
}

extern "C" lutq_status lutq_matmul_pairs(const void* X, const void* packed, const void* scales, const void* codebook,
                                         int group_size, int64_t M, int64_t N, int64_t K,
                                         lutq_dtype dtype, void* Y, void* workspace, size_t workspace_bytes,
                                         void* stream) {
    return matmul_sliced(X, packed, scales, codebook, 4, group_size, M, N, K, dtype, Y, workspace, workspace_bytes,
                         stream, nullptr, false, false, true);
}

extern "C" lutq_status lutq_matmul_quads(const void* X, const void* packed, const void* scales, const void* codebook,
                                         int group_size, int64_t M, int64_t N, int64_t K,
                                         lutq_dtype dtype, void* Y, void* workspace, size_t workspace_bytes,
                                         void* stream) {
    return matmul_sliced(X, packed, scales, codebook, 2, group_size, M, N, K, dtype, Y, workspace, workspace_bytes,
                         stream, nullptr, false, false, true);
}

namespace {

// Device address of this device's copy of `scratch`, looked up once per device with that device current.
// (In host code the array's name is only a handle for this lookup, never an address to hand to a kernel.)
lutq_status static_scratch(void** out) {
    static std::mutex mu;
    static void* ptr[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return LUTQ_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LUTQ_ERR_DEVICE;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return LUTQ_OK;
}

}  // namespace

extern "C" lutq_status lutq_matmul_static(const void* X, const void* packed, const void* scales, const void* lut,
                                          int bits, int group_size, int64_t M, int64_t N, int64_t K,
                                          lutq_dtype dtype, void* Y, void* stream, const lutq_plan* plan) {
    void* ws = nullptr;
    const lutq_status st = static_scratch(&ws);
    if (st != LUTQ_OK) return st;
    return matmul_sliced(X, packed, scales, lut, bits, group_size, M, N, K, dtype, Y, ws, LUTQ_STATIC_SCRATCH_BYTES,
                         stream, plan, false, true);
}

extern "C" lutq_status lutq_matmul(const void* X, const void* packed, const void* scales, const void* lut,
                                   int bits, int group_size, int64_t M, int64_t N, int64_t K, lutq_dtype dtype,
                                   void* Y, void* workspace, size_t workspace_bytes, void* stream) {
    return lutq_matmul_plan(X, packed, scales, lut, bits, group_size, M, N, K, dtype, Y, workspace,
                            workspace_bytes, stream, nullptr);
}

extern "C" int lutq_calib_matmul_trace(const void* X, const void* packed, const void* scales, const void* lut,
                                       int bits, int group_size, int64_t M, int64_t N, int64_t K, int dtype,
                                       void* Y, void* workspace, size_t workspace_bytes, void* stream,
                                       const lutq_plan* plan, void* trace, size_t trace_bytes, int* workgroups) {
    if (!trace || !workgroups) return LUTQ_ERR_NULL;
    if (dtype != LUTQ_F16 && dtype != LUTQ_BF16) return LUTQ_ERR_DTYPE;
    Prepared q{};
    lutq_status st = prepare_matmul(X, packed, scales, lut, bits, group_size, M, N, K, (lutq_dtype)dtype, Y, workspace,
                                    workspace_bytes, plan, false, 0, &q);
    if (st != LUTQ_OK) return st;
    if (q.queue) {
        if (bits != 4 || (group_size != 64 && group_size != 128)) return LUTQ_ERR_PLAN;
        const int groups = q.dp.G;
        if (trace_bytes < (size_t)groups * kTraceWaves * kTraceStamps * sizeof(unsigned long long) || (reinterpret_cast<uintptr_t>(trace) & 7u))
            return LUTQ_ERR_WORKSPACE;
        q.dp.trace = static_cast<unsigned long long*>(trace);
        *workgroups = groups;
        const hipError_t e = launch_decode_trace(dtype == LUTQ_BF16, group_size, q.r, q.dp, q.queue_lds, static_cast<hipStream_t>(stream));
        return e == hipSuccess ? LUTQ_OK : LUTQ_ERR_DEVICE;
    }
    // measurement builds exist for the instances the M <= 4 plans of 4-bit weights use
    if (bits != 4 || q.mb != 1 || q.xm != 4 || !q.sch || !q.wide || q.stages != 2 || q.xsh || q.r > 2 ||
        (group_size != 64 && group_size != 128))
        return LUTQ_ERR_PLAN;
    if (trace_bytes < (size_t)q.p.G * kTraceWaves * kTraceStamps * sizeof(unsigned long long) || (reinterpret_cast<uintptr_t>(trace) & 7u))
        return LUTQ_ERR_WORKSPACE;
    q.p.trace = static_cast<unsigned long long*>(trace);
    *workgroups = q.p.G;
    const hipError_t e = launch_matmul_trace(dtype == LUTQ_BF16, group_size, q.r, q.p, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LUTQ_OK : LUTQ_ERR_DEVICE;
}

namespace {

// Candidate work decompositions of lutq_tune: the default plan first, then every combination of row
// blocks per wave, teams, waves per team, grid (one workgroup per set of row groups, or 1/2, 1, 2, 4
// workgroups per compute unit with the K range cut where they do not divide the tiles) and pipeline
// depth that passes the ranges of lutq_plan.  Combinations without a kernel instance are rejected by
// lutq_matmul_plan when they are tried.
std::vector<lutq_plan> tune_candidates(int bits, int group_size, int64_t M, int64_t N, int64_t K, lutq_dtype dtype,
                                       int cus) {
    std::vector<lutq_plan> out;
    auto push_unique = [&](const lutq_plan& c) {
        for (const lutq_plan& o : out)
            if (o.row_blocks_per_wave == c.row_blocks_per_wave && o.grid == c.grid &&
                o.waves_per_workgroup == c.waves_per_workgroup && o.tiles_in_flight == c.tiles_in_flight &&
                o.row_groups_per_workgroup == c.row_groups_per_workgroup && o.scheduling == c.scheduling &&
                o.tiles_per_item == c.tiles_per_item)
                return;
        out.push_back(c);
    };
    lutq_plan def;
    if (lutq_plan_default(bits, group_size, M, N, K, dtype, &def) == LUTQ_OK) out.push_back(def);
    const int64_t nb = N / 16, kt = K / tile_k(bits);
    if (M <= 4 && (K / group_size) % 8 == 0) {
        // work-queue plans with uneven shares: one workgroup per compute unit (or per two), R = 1
        if (nb % cus != 0 && nb > cus)
            for (int g : {cus, cus / 2})
                if (g >= 1 && nb / g <= 64)
                    for (int nw : {8, 12, 16})
                        for (int it : {2, 4, 8})
                            if (kt % it == 0) push_unique(lutq_plan{1, g, nw, 2, (int)(nb / g), LUTQ_SCHED_QUEUE, it});
        // work-queue plans: row blocks per workgroup = every divisor of N/16 that leaves between half a
        // workgroup and four per compute unit, as R = 1 or 2, 8 to 16 waves, items of 2, 4, 8 tiles
        for (int64_t per = 1; per <= 64; ++per) {
            if (nb % per != 0) continue;
            const int64_t g = nb / per;
            if (g * 2 < cus || g > 4 * (int64_t)cus) continue;
            for (int r : {1, 2}) {
                if (per % r != 0 || super_block(nb) % r != 0) continue;
                for (int nw : {8, 12, 16})
                    for (int it : {2, 4, 8})
                        if (kt % it == 0)
                            push_unique(lutq_plan{r, (int)g, nw, 2, (int)(per / r), LUTQ_SCHED_QUEUE, it});
            }
        }
    }
    if (M > 4 && nb >= cus / 2) {
        // row-streaming plans: one workgroup per compute unit (or two, or one per two), four and eight row blocks
        // side by side, all the waves the instance allows and eight
        const int mbh = M > 16 ? 2 : 1;
        for (int g : {cus, 2 * cus, cus / 2}) {
            if (g < 1 || g > nb || nb / g > 64) continue;
            for (int side : {4, 8}) {
                const int w = rows_instance_waves(bits, dtype == LUTQ_BF16, mbh, side);
                if (w == 0) continue;
                for (int nw : {w, 8})
                    if (nw <= w) push_unique(lutq_plan{side, g, nw, 2, (int)(nb / g), LUTQ_SCHED_ROWS, 0});
            }
        }
    }
    if (M > 4 && nb <= 2 * (int64_t)cus) {
        // the same with K cut into slices across workgroups: one pass per share of four or eight row blocks, grids of one
        // workgroup per compute unit, half and twice that
        const int mbh = M > 16 ? 2 : 1;
        for (int side : {4, 8}) {
            const int w = rows_instance_waves(bits, dtype == LUTQ_BF16, mbh, side);
            if (w == 0) continue;
            const int64_t shares = (nb + side - 1) / side;
            if (shares * 64 > (int64_t)kCounterBytes) continue;
            for (int64_t ks = 2; ks <= kt && shares * ks <= 2 * (int64_t)cus; ++ks) {
                if (shares * ks > kMaxGrid || (kt % ks != 0 && (kt + (kt + ks - 1) / ks - 1) / ((kt + ks - 1) / ks) != ks)) continue;
                // (small problems, whose grids stay below half the compute units, keep the two extremes)
                if (shares * ks * 2 < cus && ks != 2 && ks != kt) continue;
                for (int nw : {w, 8})
                    if (nw <= w) push_unique(lutq_plan{side, (int)(shares * ks), nw, 2, (int)(nb / shares), LUTQ_SCHED_ROWS, (int)((kt + ks - 1) / ks)});
            }
        }
    }
    for (int r : {1, 2, 4}) {
        if (super_block(nb) % r != 0) continue;
        const int64_t nrg = nb / r;
        for (int rs = 1; rs <= 16; ++rs) {
            if (nrg % rs != 0) continue;
            const int64_t sets = nrg / rs, tiles = sets * kt;
            for (int ks = 1; ks * rs <= 16; ++ks) {
                const int nw = ks * rs;
                if (nw < 4 || (nw > 8 && nw % 2 != 0)) continue;
                int64_t grids[5] = {sets, cus / 2, cus, 2 * cus, 4 * cus};
                for (int gi = 0; gi < 5; ++gi) {
                    const int64_t g = grids[gi];
                    if (g < 1 || g > tiles || g * rs > kMaxGrid) continue;
                    if (gi > 0 && g == sets) continue;
                    for (int stages : {2, 4}) {
                        push_unique(lutq_plan{r, (int)g, nw, stages, rs, LUTQ_SCHED_TEAMS, 0});
                    }
                }
            }
        }
    }
    return out;
}

}  // namespace

extern "C" lutq_status lutq_tune_candidates(int bits, int group_size, int64_t M, int64_t N, int64_t K,
                                            lutq_dtype dtype, lutq_plan* plans, int capacity, int* count) {
    if (!count || (capacity > 0 && !plans)) return LUTQ_ERR_NULL;
    lutq_status st = check_problem(bits, group_size, N, K);
    if (st != LUTQ_OK) return st;
    if (M < 1 || M > kMaxRows) return LUTQ_ERR_SHAPE;
    if (dtype != LUTQ_F16 && dtype != LUTQ_BF16) return LUTQ_ERR_DTYPE;
    DeviceInfo di = device_info();
    if (!di.ok) return LUTQ_ERR_DEVICE;
    const std::vector<lutq_plan> c = tune_candidates(bits, group_size, M, N, K, dtype, di.cus);
    *count = (int)c.size();
    for (int i = 0; i < (int)c.size() && i < capacity; ++i) plans[i] = c[i];
    return LUTQ_OK;
}

extern "C" lutq_status lutq_tune(const void* X, const void* const* packed, const void* const* scales, int ring,
                                 const void* lut, int bits, int group_size, int64_t M, int64_t N, int64_t K,
                                 lutq_dtype dtype, void* Y, void* workspace, size_t workspace_bytes, void* stream,
                                 int reps, lutq_plan* best, float* best_us) {
    if (!packed || !scales || !best) return LUTQ_ERR_NULL;
    if (ring < 1 || reps < 1) return LUTQ_ERR_SHAPE;
    for (int i = 0; i < ring; ++i)
        if (!packed[i] || !scales[i]) return LUTQ_ERR_NULL;
    lutq_plan def;
    lutq_status st = lutq_plan_default(bits, group_size, M, N, K, dtype, &def);
    if (st != LUTQ_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the default plan validates every other argument; its launches also bring the clocks up
    int next = 0;
    auto run = [&](const lutq_plan& c, int n) {
        lutq_status r = LUTQ_OK;
        for (int i = 0; i < n && r == LUTQ_OK; ++i) {
            r = lutq_matmul_plan(X, packed[next], scales[next], lut, bits, group_size, M, N, K, dtype, Y, workspace,
                                 workspace_bytes, s, &c);
            next = next + 1 == ring ? 0 : next + 1;
        }
        return r;
    };
    st = run(def, 1);
    if (st != LUTQ_OK) return st;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess) return LUTQ_ERR_DEVICE;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return LUTQ_ERR_DEVICE; }
    auto cleanup = [&](lutq_status r) { (void)hipEventDestroy(e0); (void)hipEventDestroy(e1); return r; };
    // microseconds per launch of n launches of plan c; negative if the plan has no instance
    auto time_plan = [&](const lutq_plan& c, int n, float* us) {
        lutq_status r = run(c, 2);
        if (r != LUTQ_OK) return r;
        if (hipEventRecord(e0, s) != hipSuccess) return LUTQ_ERR_DEVICE;
        r = run(c, n);
        if (r != LUTQ_OK) return r;
        float ms = 0.f;
        if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
            return LUTQ_ERR_DEVICE;
        *us = ms * 1000.f / (float)n;
        return LUTQ_OK;
    };
    float us = 0.f;
    for (float spent = 0.f; spent < 50000.f; spent += us * 20.f)          // about 50 ms of load before timing
        if ((st = time_plan(def, 20, &us)) != LUTQ_OK) return cleanup(st);
    DeviceInfo di = device_info();
    if (!di.ok) return cleanup(LUTQ_ERR_DEVICE);
    const std::vector<lutq_plan> cands = tune_candidates(bits, group_size, M, N, K, dtype, di.cus);
    // first pass: a few launches each; second pass: the best eight at full length
    std::vector<std::pair<float, int>> order;
    const int quick = reps < 8 ? reps : 8;
    for (int i = 0; i < (int)cands.size(); ++i) {
        st = time_plan(cands[i], quick, &us);
        if (st == LUTQ_ERR_PLAN) continue;
        if (st != LUTQ_OK) return cleanup(st);
        order.emplace_back(us, i);
        if (env_switches().verbose == 2)
            std::fprintf(stderr, "lutq_tune: quick R=%d grid=%d waves=%d stages=%d teams=%d: %.2f us\n",
                         cands[i].row_blocks_per_wave, cands[i].grid, cands[i].waves_per_workgroup,
                         cands[i].tiles_in_flight, cands[i].row_groups_per_workgroup, us);
    }
    if (order.empty()) return cleanup(LUTQ_ERR_PLAN);
    std::sort(order.begin(), order.end());
    bool have_default = false;
    const int finalists = (int)order.size() < 8 ? (int)order.size() : 8;
    for (int j = 0; j < finalists; ++j) have_default = have_default || order[j].second == 0;
    // final pass: three rounds over the finalists in alternating order, the minimum per plan counts
    // (clocks drift over a run of this length, so a single pass would favour whoever is timed first)
    std::vector<int> fin;
    for (int j = 0; j < finalists; ++j) fin.push_back(order[j].second);
    if (!have_default) fin.push_back(0);
    std::vector<float> tmin(fin.size(), 0.f);
    for (int round = 0; round < 3; ++round)
        for (size_t jj = 0; jj < fin.size(); ++jj) {
            const size_t j = (round & 1) ? fin.size() - 1 - jj : jj;
            if ((st = time_plan(cands[fin[j]], reps, &us)) != LUTQ_OK) return cleanup(st);
            if (round == 0 || us < tmin[j]) tmin[j] = us;
        }
    float best_time = 0.f;
    int best_i = -1;
    for (size_t j = 0; j < fin.size(); ++j) {
        const int i = fin[j];
        if (env_switches().verbose)
            std::fprintf(stderr, "lutq_tune: %s R=%d grid=%d waves=%d stages=%d teams=%d: %.2f us\n", i == 0 ? "default" : "candidate",
                         cands[i].row_blocks_per_wave, cands[i].grid, cands[i].waves_per_workgroup,
                         cands[i].tiles_in_flight, cands[i].row_groups_per_workgroup, tmin[j]);
        if (best_i < 0 || tmin[j] < best_time) { best_time = tmin[j]; best_i = i; }
    }
    *best = cands[best_i];
    if (best_us) *best_us = best_time;
    return cleanup(LUTQ_OK);
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
    hipError_t e = pick_dequant(bits, dtype)(group_size, p, (int)grid, lut_bytes(bits, dtype == LUTQ_BF16, p.log2c) + 2048,
                                             static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LUTQ_OK : LUTQ_ERR_DEVICE;
}
