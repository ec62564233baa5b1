// The fused kernel for decode-sized batches (M <= 4) with a work queue inside the workgroup.
//
// What is computed is that of matmul_kernel (Algorithm 1 of the paper: table to on-chip memory, stream
// the restructured weights, combine bit-slices, vectorised lookup + group scale, matrix instruction).
// What differs is how the work of one compute unit is dealt to its wavefronts (the paper's Section 3.3
// concern, here inside a workgroup instead of across them):
//
//   * A workgroup owns A consecutive row groups (a row group = R 16-row blocks) over the whole of K and
//     nothing else, so no partial sum ever leaves it (no cross-workgroup fix-up).  Where the row groups
//     do not divide over the workgroups the first `extra` workgroups own A + 1: better a few compute
//     units with one more row group than every output tile cut in two and put together again.
//   * Its work is cut into items: (row group a, IT consecutive K tiles).  Wave w starts with item w;
//     whenever a wave finishes an item it takes the next one from a counter in LDS.  A wave that the
//     hardware favours (the issue arbiter serves old waves first, and 14 waves do not divide over 4
//     SIMDs) simply takes more items, so all waves finish within one item of each other; with a static
//     split the slowest wave of a compute unit ends 20 % after the fastest.
//   * The result must not depend on who computed what: every item's partial sums go to the item's own
//     slot in LDS, and after a barrier each output is summed over its items in K order.  Together with
//     the fixed order inside an item that makes Y bit-reproducible whatever the timing.
//   * The prologue is kept short: on this hardware a SIMD issues one scalar (and one vector) instruction
//     per four cycles whichever of its waves it comes from, so the scalar set-up of four waves per SIMD
//     runs back to back and every instruction of it delays the fourth wave's first load by four times
//     its own issue time.  Everything that is uniform over the launch is therefore computed on the host.
//
// Activations use the packed layout for M <= 4 (one 128-bit load covers four 32-wide K steps: lane i
// holds row i % 4 of step i / 4; four accumulators folded by three row rotations per item).
//
// RLUT (one table per output row, Section 2.3's tables at the output-channel level): the four lanes that
// work on a row share one copy of that row's table, so a row block's tables are 16 copies (16 KiB at 4
// bits) instead of 64, and the tables of ALL the workgroup's row blocks are built once, before the K
// loop: a launch then costs what the shared-table launch costs plus the larger build and one more
// instruction per lookup (the entry stride is no longer the 256 bytes that one byte permute addresses;
// two lanes of a row that read different entries can meet in a bank).
#pragma once

#include <type_traits>

#include "lutq_matmul_kernel.hpp"

namespace lutq {

struct DecodeParams {
    const uint16_t* X;        // [M, K]
    const uint8_t* packed;
    const uint16_t* scales;   // [N, SG]
    const uint16_t* lut;
    uint16_t* Y;              // [M, N]
    uint32_t packed_bytes, scale_bytes, x_bytes;
    int M, N, K;
    int SG2;                  // bytes of one row of scales (2 K / group)
    int SBL;                  // log2 of the row blocks per super-block of the packed layout (R divides it)
    uint32_t tile_stride;     // packed bytes from K tile kt to kt + 1 of one row block (tile bytes << SBL)
    uint32_t sblock_bytes;    // packed bytes of one super-block
    int A;                    // row groups per workgroup ...
    int extra;                // ... plus one more in workgroups 0 .. extra - 1
    int C;                    // items per row group (K tiles per row block = C * IT)
    int IT;                   // K tiles per item, a multiple of the pipeline depth
    int NW;                   // waves per workgroup
    int G;                    // workgroups
    uint32_t a_magic;         // floor(2^32 / A) (0xffffffff for A = 1), see div_magic
    uint32_t a1_magic;        // the same for A + 1
    int lut_ltpe;             // log2 of the threads that build one table row together
    int slot_off;             // LDS byte offset of the item slots
    int NG, GL;               // final reduction: NG groups of GL consecutive items per output (NG * GL >= C)
    uint32_t o_magic;         // floor(2^32 / (A * R * 64))
    uint32_t o1_magic;        // floor(2^32 / ((A + 1) * R * 64))
    int tab_total;            // RLUT: LDS bytes of all the row blocks' tables (the other areas follow)
    int NB;                   // waves 0 .. NB - 1 build the shared table; the others wait for it before their first loads
    unsigned long long* trace;   // TRACE instances only
};

// LDS of one launch: [table, 256-byte entry stride][queue counter, 256 bytes][1 KiB scale-chunk area per wave]
// [one slot per item: R x 64 floats (16 rows x 4 activation rows)]
template <int BITS>
__host__ __device__ constexpr int decode_scale_off() { return lut_row_table_bytes<BITS>() + 256; }
template <int BITS>
__host__ __device__ constexpr int decode_slot_off(int nw) { return decode_scale_off<BITS>() + nw * 1024; }
template <int BITS>
__host__ __device__ constexpr int decode_lds_bytes(int nw, int items, int r) { return decode_slot_off<BITS>(nw) + items * r * 256; }

// Instances that exist: R = 1 or 2, except 3-bit bf16 at R = 2 (two bit-slices per tile and the widened
// table's lookup ring do not fit 128 registers next to two row blocks' accumulators).
__host__ __device__ constexpr bool decode_instance_exists(int bits, bool bf16, int r) {
    return (r == 1 || r == 2) && !(bits == 3 && bf16 && r == 2);
}

template <int BITS, int GROUP, int R, typename DT, int P, bool TRACE = false, bool RLUT = false>
__global__ __launch_bounds__(1024) void decode_kernel(const DecodeParams p) {
    static_assert(!RLUT || R == 1, "per-row tables: one row block per row group");
    using Gm = Geo<BITS>;
    constexpr int TK = Gm::TK, STEPS = Gm::STEPS, TILE_BYTES = Gm::TILE_BYTES;
    constexpr int TPS = GROUP > TK ? GROUP / TK : 1;   // tiles that share one scale
    constexpr int NS = GROUP > TK ? 1 : TK / GROUP;    // scales per tile per row
    constexpr int SPG = GROUP / 32;                    // steps per group
    constexpr int TPC = 8 * TPS / NS;                  // tiles covered by one 16-byte scale chunk
    constexpr int LOG2C = perm_log2_copies<BITS, DT>();
    constexpr int U = STEPS * R;                       // (step, row block) items of one tile
    constexpr int D = U < 4 ? U : 4;                   // table reads kept in flight ahead of their use
    constexpr int XL = STEPS / 4;                      // activation loads per tile (four steps each)

    unsigned long long tr[kTraceStamps];
    auto stamp = [&](int i) {
        if constexpr (TRACE) {
            if (tr[i] == 0) tr[i] = wall_clock64();
        }
    };
    if constexpr (TRACE) {
#pragma unroll
        for (int i = 0; i < kTraceStamps; ++i) tr[i] = 0;
        stamp(kTraceStart);
    }
    asm volatile("" ::"s"(p.X), "s"(p.packed), "s"(p.scales), "s"(p.lut), "s"(p.Y), "s"(p.packed_bytes), "s"(p.scale_bytes),
                 "s"(p.x_bytes), "s"(p.M), "s"(p.N), "s"(p.K), "s"(p.SG2), "s"(p.SBL), "s"(p.tile_stride), "s"(p.sblock_bytes),
                 "s"(p.A), "s"(p.C), "s"(p.IT), "s"(p.NW), "s"(p.a_magic), "s"(p.lut_ltpe), "s"(p.slot_off), "s"(p.NG), "s"(p.GL),
                 "s"(p.o_magic), "s"(p.extra), "s"(p.a1_magic), "s"(p.o1_magic), "s"(p.tab_total), "s"(p.NB));
    stamp(kTraceArgs);

    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15;                // row inside a 16-row block (A side)
    char* lut = smem;
    const int table_bytes = RLUT ? p.tab_total : lut_row_table_bytes<BITS>();
    uint32_t* queue = reinterpret_cast<uint32_t*>(smem + table_bytes);
    char* sc_lds = smem + table_bytes + 256 + wave * 1024;
    float* slots = reinterpret_cast<float*>(smem + p.slot_off);

    const bool big = (int)blockIdx.x < p.extra;        // this workgroup owns one row group more
    const int A = p.A + (big ? 1 : 0);
    const int rg0 = (int)blockIdx.x * p.A + ((int)blockIdx.x < p.extra ? (int)blockIdx.x : p.extra);   // first row group

    // Sixteen waves' first loads queue up in the compute unit's address unit, and the table is not complete before
    // the last wave has got its loads out and joined the build: with sixteen waves only the first NB = 8 build
    // the table, and the others meet them at the barrier BEFORE they ask for anything.  The builders' loads then go
    // out unhindered, the table stands earlier, and the later waves start from a built table.  (Every wave passes
    // the one barrier exactly once, here or after the build.)
    const bool builder = RLUT || wave < p.NB;
    if (!builder) __syncthreads();

    // the table's values are asked for first: they are needed first
    LutSeed lut_seed{};
    uint32_t rowtab_raw[2] = {0, 0};
    if constexpr (RLUT) {
        // the raw tables of the workgroup's rows (consecutive rows: one contiguous range), two words per thread
        const rsrc_t rT = make_rsrc(p.lut, (uint32_t)p.N * (uint32_t)((1 << BITS) * 2));
        const int words = A * (rowlut16_stage_bytes<BITS>() / 4);
        const uint32_t tbase = (uint32_t)rg0 * (uint32_t)rowlut16_stage_bytes<BITS>();
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int i = tid + k * p.NW * 64;
            rowtab_raw[k] = __builtin_amdgcn_raw_buffer_load_b32(rT, i < words ? tbase + 4u * (uint32_t)i : kOutOfRange, 0, kAuxNone);
        }
    } else {
        lut_seed = lut_fetch<BITS>(p.lut, tid, p.lut_ltpe);
    }
    __builtin_amdgcn_sched_barrier(0);
    const LutAddr la = make_lut_addr<BITS, DT>(lut, RLUT ? 4 : LOG2C, lane);

    const rsrc_t rW = make_rsrc(p.packed, p.packed_bytes);
    const rsrc_t rS = make_rsrc(p.scales, p.scale_bytes);
    const rsrc_t rX = make_rsrc(p.X, p.x_bytes);

    // activations: lane i of a 16-lane row holds row i % 4 of K step i / 4 of the load's four steps;
    // rows m >= M start beyond the buffer and read as zero
    const uint32_t xlane = ((uint32_t)(li & 3) * (uint32_t)p.K + 32u * (uint32_t)(li >> 2) + 8u * (uint32_t)(lane >> 4)) * 2u;
    const uint32_t wlane = 16u * lane;
    // scale chunks: lane l < 16 R fetches 16 bytes of row l of the row group
    const uint32_t clane = lane < 16 * R ? (uint32_t)lane * (uint32_t)p.SG2 : kOutOfRange;
    const uint32_t a_magic = big ? p.a1_magic : p.a_magic;
    const int nitems = A * p.C;

    // the queue hands out items NW, NW + 1, ...: items 0 .. NW - 1 are the waves' first ones
    if (tid == 0) *queue = (uint32_t)p.NW;
    const uint32_t queue_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint32_t*)queue;

    struct Stage {
        WFrag<BITS> w[R];
        u32x4 chunk;                       // 8 consecutive scales of row `lane` of the row group
        u32x4 x[XL];
    };
    // where an item's tiles are: packed-weight offset of its first tile, scale offset of its row
    // group, first K tile
    // (an item beyond the last one gets bases of exactly 2 GiB: every offset formed from them stays out
    // of range without wrapping, and no branch is needed -- with a branch the compiler duplicates the
    // loads on both paths and then waits for all outstanding loads where the paths join)
    struct Item { uint32_t wbase, sbase, xbase; int kt0; uint32_t tab; };   // tab (RLUT): LDS offset of the row block's tables
    auto locate = [&](int item) -> Item {
        Item it;
        const int c = div_magic(item, a_magic, A);        // items are numbered K-major: item = c * A + a
        const int a = item - c * A;
        const int rb0 = (rg0 + a) * R;
        const bool in = item < nitems;
        it.kt0 = c * p.IT;
        const uint32_t wb = (uint32_t)(rb0 >> p.SBL) * p.sblock_bytes + (uint32_t)(rb0 & ((1 << p.SBL) - 1)) * TILE_BYTES
                          + (uint32_t)it.kt0 * p.tile_stride;
        it.wbase = in ? wb : kOutOfRange;
        it.sbase = in ? (uint32_t)rb0 * 16u * (uint32_t)p.SG2 : kOutOfRange;
        it.xbase = in ? (uint32_t)it.kt0 * (TK * 2) : kOutOfRange;
        it.tab = RLUT && in ? (uint32_t)a * (uint32_t)rowlut16_bytes<BITS, DT>() : 0u;
        return it;
    };
    // loads of tile j of an item (K tile kt0 + j); an item beyond the last one has out-of-range bases.
    // The weights and the rest (scale chunk, activations) are separate so that the prologue can ask for
    // the weights alone: every 128-bit load occupies the compute unit's address unit for 16 cycles
    // whatever it fetches, and sixteen waves' first loads queue up there, so the loads that have to
    // come all the way from HBM go first and the others follow once the table is built.
    auto load_weights = [&](Stage& st, const Item& it, int j) {
        const uint32_t tw = it.wbase + (uint32_t)j * p.tile_stride;
#pragma unroll
        for (int r = 0; r < R; ++r) load_wfrag<BITS>(st.w[r], rW, tw + r * TILE_BYTES, lane);
    };
    // (`always`: issue the scale-chunk load whether or not a chunk starts at this tile, so that the number
    // of loads between the table fetch and the wait for it is the same on every path and the wait
    // counts the table's loads exactly)
    auto load_rest = [&](Stage& st, const Item& it, int j, auto always) {
        const int kt = it.kt0 + j;
        const bool first = (kt % TPC) == 0 || j == 0;
        const uint32_t tc = first ? it.sbase + (uint32_t)(kt / TPC) * 16u : kOutOfRange;
        if (decltype(always)::value || first) st.chunk = __builtin_amdgcn_raw_buffer_load_b128(rS, tc + clane, 0, kAuxNone);
        const uint32_t tx = it.xbase + (uint32_t)j * (TK * 2);
#pragma unroll
        for (int x = 0; x < XL; ++x) st.x[x] = __builtin_amdgcn_raw_buffer_load_b128(rX, tx + xlane + 256u * x, 0, kAuxNone);
    };
    auto load_stage = [&](Stage& st, const Item& it, int j) {
        load_weights(st, it, j);
        load_rest(st, it, j, std::false_type{});
    };

    f32x4 acc[R][4];
    auto compute_stage = [&](const Stage& st, int kt, int j, uint32_t tab) {
        LutAddr la_item = la;
        if constexpr (RLUT) la_item.lane_base += tab;
        constexpr bool PERM = !RLUT;
        ScaleWords<NS> sw[R];
        if ((kt % TPC) == 0 || j == 0) {
            // a new chunk: every lane parks its row's 8 scales in LDS, then each lane picks the scales
            // of its own rows (LDS operations of one wave complete in order)
            asm volatile("" ::: "memory");
            *reinterpret_cast<u32x4*>(sc_lds + 16 * lane) = st.chunk;
            asm volatile("" ::: "memory");
        }
        const char* src = sc_lds + 16 * li + ((kt % TPC) / TPS) * (NS * 2);
#pragma unroll
        for (int r = 0; r < R; ++r) lds_load_scales<NS>(sw[r], src + 256 * r);
        Raw<BITS, DT> raw[D];
#pragma unroll
        for (int u = 0; u < D; ++u) raw[u] = lookup_step<BITS, DT, PERM>(st.w[u % R], u / R, la_item);
        __builtin_amdgcn_sched_barrier(0);
        u32x4 a[2];
#pragma unroll
        for (int u = 0; u <= U; ++u) {
            if (u < U) {
                const int s = u / R, r = u % R;
                const ScaleReg<DT> sc = scale_of<DT, NS>(sw[r], s / SPG);
                a[u & 1] = scale4<BITS, DT>(raw[u % D], sc);
                __builtin_amdgcn_sched_barrier(0);
                if (u + D < U) {
                    raw[u % D] = lookup_step<BITS, DT, PERM>(st.w[(u + D) % R], (u + D) / R, la_item);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (u > 0) {
                const int s = (u - 1) / R, r = (u - 1) % R;
                acc[r][s % 4] = mfma16x16x32<DT>(a[(u - 1) & 1], st.x[s / 4], acc[r][s % 4]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    int item = wave;
    Item cur = locate(item);
    Stage st[P];
#pragma unroll
    for (int q = 0; q < P; ++q) {
        load_weights(st[q], cur, q);
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int q = 0; q < P; ++q) {
        load_rest(st[q], cur, q, std::true_type{});
        __builtin_amdgcn_sched_barrier(0);
    }
    stamp(kTraceIssued);
    if constexpr (RLUT) {
        // the raw tables go to LDS -- into the item slots' area, which nothing uses before the K loop -- and
        // the copies are built from there, while the first tiles are in flight
        const int words = A * (rowlut16_stage_bytes<BITS>() / 4);
        char* stage = reinterpret_cast<char*>(slots);
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int i = tid + k * p.NW * 64;
            if (i < words) *reinterpret_cast<uint32_t*>(stage + 4 * i) = rowtab_raw[k];
        }
        __syncthreads();
        rowlut16_build<BITS, DT>(lut, stage, A, tid, p.NW * 64);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
    } else if (builder) {
        // the table is built while the first tiles are in flight (its own reads were issued before them)
        LutSeed seed = lut_seed;
        asm volatile("" : "+v"(seed.w[0]), "+v"(seed.w[1]), "+v"(seed.w[2]), "+v"(seed.w[3]));
        lut_build<BITS, DT>(lut, seed, (int)(reinterpret_cast<uintptr_t>(p.lut) >> 1) & 1, LOG2C, tid, p.lut_ltpe);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
    }
    stamp(kTraceTable);

    while (item < nitems) {
        // the next item is taken now and needed when this item's last tiles are being computed
        // (one lane's LDS add, written out: left to the compiler the `if (lane == 0)` around it ends with a
        // wait for the returned value, which would stall every item by an LDS round trip)
        uint32_t nextv;
        {
            uint64_t saved_exec;
            asm volatile("s_mov_b64 %1, exec\n\ts_mov_b64 exec, 1\n\tds_add_rtn_u32 %0, %2, %3\n\ts_mov_b64 exec, %1"
                         : "=&v"(nextv), "=&s"(saved_exec) : "v"(queue_addr), "v"(1u) : "memory");
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int a = 0; a < 4; ++a) acc[r][a] = f32x4{0.f, 0.f, 0.f, 0.f};
        int j = 0;
        for (; j + P < p.IT; j += P) {
#pragma unroll
            for (int q = 0; q < P; ++q) {
                compute_stage(st[q], cur.kt0 + j + q, j + q, cur.tab);
                __builtin_amdgcn_sched_barrier(0);
                stamp(kTraceFirstTile);
                load_stage(st[q], cur, j + q + P);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // last P tiles of the item: the prefetches go to the first tiles of the next item
        __builtin_amdgcn_s_waitcnt(0xc07f);                 // lgkmcnt(0): the counter value has arrived
        asm volatile("" : "+v"(nextv));
        const int next = __builtin_amdgcn_readfirstlane((int)nextv);
        const Item nxt = locate(next);
#pragma unroll
        for (int q = 0; q < P; ++q) {
            compute_stage(st[q], cur.kt0 + j + q, j + q, cur.tab);
            __builtin_amdgcn_sched_barrier(0);
            stamp(kTraceFirstTile);
            load_stage(st[q], nxt, q);
            __builtin_amdgcn_sched_barrier(0);
        }
        // fold the four step positions (columns 4 j .. 4 j + 3 of accumulator j move to columns 0 .. 3)
        // and hand the item's sums over: lane (o, i < 4) holds rows 4 o .. 4 o + 3 of activation row i
        float* slot = slots + (size_t)item * (R * 64);
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int jj = 1; jj < 4; ++jj) {
                const u32x4 t = rotate_rows(__builtin_bit_cast(u32x4, acc[r][jj]), 4 * jj);
                acc[r][0] += __builtin_bit_cast(f32x4, t);
            }
            if (li < 4) *reinterpret_cast<f32x4*>(slot + r * 64 + li * 16 + 4 * (lane >> 4)) = acc[r][0];
        }
        item = next;
        cur = nxt;
    }
    stamp(kTraceLoopDone);
    __syncthreads();
    stamp(kTraceReduced);
    // Every output is the sum of its C items: output o = ((a R + r) 4 + m) 16 + n of the workgroup lives
    // at float o of the slots of items c A + a.  The items of an output are cut into NG groups of GL
    // consecutive ones (both fixed by the launch, not by the timing); thread (g, o) adds group g in K
    // order, then thread o adds the group sums in order: the same tree on every run.
    const int outputs = A * R * 64;
    const uint32_t o_magic = big ? p.o1_magic : p.o_magic;
    float* gsum = reinterpret_cast<float*>(lut);        // the table is no longer needed
    if (p.NG > 1) {
        for (int idx = tid; idx < outputs * p.NG; idx += p.NW * 64) {
            const int g = div_magic(idx, o_magic, outputs);
            const int o = idx - g * outputs;
            const int c0 = g * p.GL, c1 = (c0 + p.GL < p.C) ? c0 + p.GL : p.C;
            const float* src = slots + o;
            float sum = 0.f;
#pragma unroll 8
            for (int c = c0; c < c1; ++c) sum += src[(size_t)c * outputs];
            gsum[idx] = sum;
        }
        __syncthreads();
    }
    for (int o = tid; o < outputs; o += p.NW * 64) {
        float sum = 0.f;
        if (p.NG > 1) {
#pragma unroll 8
            for (int g = 0; g < p.NG; ++g) sum += gsum[g * outputs + o];
        } else {
            const float* src = slots + o;
#pragma unroll 8
            for (int c = 0; c < p.C; ++c) sum += src[(size_t)c * outputs];
        }
        const int n16 = o & 15, m = (o >> 4) & 3, rb = o >> 6;           // rb = a R + r
        if (m < p.M) {
            const size_t at = (size_t)m * p.N + (size_t)(rg0 * R + rb) * 16 + n16;
            if constexpr (std::is_same<DT, F16>::value) {
                const _Float16 h = (_Float16)sum;
                p.Y[at] = __builtin_bit_cast(uint16_t, h);
            } else {
                const __bf16 h = (__bf16)sum;
                p.Y[at] = __builtin_bit_cast(uint16_t, h);
            }
        }
    }
    if constexpr (TRACE) {
        __builtin_amdgcn_s_waitcnt(0);
        stamp(kTraceEnd);
        if (p.trace && lane == 0) {
            unsigned long long* o = p.trace + ((size_t)blockIdx.x * kTraceWaves + wave) * kTraceStamps;
#pragma unroll
            for (int i = 0; i < kTraceStamps; ++i) o[i] = tr[i];
        }
    }
}

}  // namespace lutq
