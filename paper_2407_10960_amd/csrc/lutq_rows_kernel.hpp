// The fused kernel for 5 to 32 activation rows on matrices with several row blocks per compute unit, and for 33 to 64
// rows at 4 bits (three or four blocks of sixteen rows; the activations then come from an operand-order copy).
//
// What is computed is that of matmul_kernel (Algorithm 1 of the paper).  The loop nest is turned round:
// from five rows up the activations are as large a stream as the weights (M x 128 x 2 bytes per 1 KiB
// weight tile at 4 bits: one to eight times the weights for M = 4 .. 32), so this kernel holds the
// activations still and streams weights past them:
//
//   * A workgroup owns A consecutive 16-row blocks over the whole of K (the first `extra` workgroups one
//     more), nothing else: no partial sum leaves it.
//   * Its waves split K.  For each of its K tiles a wave loads the tile's activations once -- all M rows,
//     as B operands of the matrix instruction, into registers -- and then walks the workgroup's row
//     blocks: one 1 KiB weight tile per row block, dequantised through the table and multiplied into
//     that row block's accumulators.  Up to AMAX row blocks are accumulated side by side (AMAX x MB x 4
//     registers); a workgroup with more walks them in passes of AMAX.
//   * So an activation fragment is fetched once per AMAX weight tiles instead of once per tile or per
//     pair of tiles, no activation goes through LDS, and there is no barrier inside the K loop: the waves
//     run out of step and cover each other's memory and table-lookup latencies.
//   * After a pass the waves' accumulators are added in wave order through LDS, a few row blocks per
//     round, and written out: bit-reproducible.
//
//   * K slices (matrices with fewer row blocks than would keep every compute unit busy): KS workgroups share a
//     workgroup's row blocks (at most AMAX: one pass) and take a slice of K each (as even as whole tiles allow), so that a compute unit reads only
//     its slice of the activations.  Each writes its sums (fp32, per row block and block of sixteen rows of M) to its
//     own slot in global memory and, when all of them are stored, bumps the share's arrival counter once; whichever
//     workgroup arrives last adds the KS slots in slice order, its own included, and writes Y: nobody waits for anybody, and the result does not
//     depend on who was last.  (Moved with agent-scope atomic loads and stores, ordered by completion: the stores are
//     acknowledged before the counter is bumped, and the loads are issued after the counter value that proves the
//     workgroup is last has come back -- the protocol of matmul_kernel's fix-up.)
//
//   * The scales of a pass's row blocks (consecutive rows: one contiguous range) are copied into LDS when
//     the pass begins, 16 bytes per lane, and read from there per (tile, row block): a 2- to 16-byte read
//     per lane from global memory would touch sixteen cache lines per instruction for one line's worth of
//     weights.
#pragma once

#include <type_traits>

#include "lutq_matmul_kernel.hpp"

namespace lutq {

struct RowsParams {
    const uint16_t* X;        // [M, K]; MB > 2: the operand-order copy (rows_xop_kernel), KT x STEPS x MB fragments of 1 KiB
    const uint8_t* packed;
    const uint16_t* scales;   // [N, SG]
    const uint16_t* lut;
    uint16_t* Y;              // [M, N]
    uint32_t packed_bytes, scale_bytes, x_bytes;
    int M, N, K;
    int KT;                   // K tiles per row block
    int SG2;                  // bytes of one row of scales
    int SBL;                  // log2 of the row blocks per super-block of the packed layout
    uint32_t tile_stride;     // packed bytes from K tile kt to kt + 1 of one row block
    uint32_t sblock_bytes;    // packed bytes of one super-block
    int A, extra;             // row blocks per workgroup; workgroups 0 .. extra - 1 own one more
    int NW;                   // waves per workgroup
    int TQ, TR;               // KT = TQ * NW + TR: wave w owns TQ (+1 if w < TR) consecutive K tiles
    int RPR;                  // row blocks reduced per round (RPR * MB * NW KiB of LDS)
    int s_units;              // 16-byte units per row of scales (SG2 / 16)
    uint32_t s_magic;         // 2^32 / s_units + 1 (unused when s_units == 1)
    int SROW;                 // bytes from row to row of the scales in LDS (SG2 + 16: sixteen rows, sixteen banks)
    int red_off;              // LDS offset of the reduction slots
    int tab_total;            // RLUT: LDS bytes of the pass's per-row tables (AMAX x sixteen copies); the scales follow
    int lut_ltpe;             // log2 of the threads that build one table row together
    int G;                    // workgroups
    int KS;                   // K slices: workgroup b works on slice b % KS of the row blocks of share b / KS (1: the whole of K)
    int TS;                   // K tiles per slice (the whole part of KT / KS); the first KSB slices have one more
    int KSB;                  // KT % KS
    int TQ1, TR1;             // TQ, TR of the slices with TS + 1 tiles
    float* slots;             // KS > 1: partial sums, one slot of AMAX x MB KiB per workgroup
    uint32_t* counters;       // KS > 1: arrivals per share, one counter per 64 bytes; zero between launches
};

// LDS of one launch: [table, 256-byte entry stride][scales of AMAX x 16 rows, SROW bytes each][RPR x MB x NW slots of 1 KiB]
// RLUT: [AMAX tables of sixteen copies][scales][raw tables of AMAX row blocks][slots]

// Registers: AMAX x MB x 4 accumulators + STEPS x MB x 4 activation operands (twice that where two tiles' are
// held) + four weight tiles in flight, the lookup ring and addresses (about 84 at 4 bits, 108 and 116 at 2 and
// 3 bits with their eight steps per tile, 28 more with a widened bf16 table, 20 more at 4 bits with eight row
// blocks side by side).  The estimate decides how many waves an instance is compiled for (4-bit fp16: M <= 16
// with four / eight row blocks side by side 114 / 149 registers, sixteen / twelve waves; M > 16 191 / 241,
// eight waves); 0 = no such instance (the registers do not hold it without spilling).
__host__ __device__ constexpr int rows_tiles_in_flight(int, int) { return 4; }   // (eight measured no faster)
// The activations of the next K tile are fetched a whole tile ahead into a second set of registers where that
// measured faster (4-bit fp16 beyond sixteen rows: 8B gate+up M = 32 21.9 -> 20.8 us); elsewhere the second set
// costs waves (twelve -> eight) or the instance, and the next tile's activations are fetched step by step
// during the tile's last row block instead.
__host__ __device__ constexpr bool rows_x_double(int bits, int mb, bool wide_table) { return bits == 4 && mb == 2 && !wide_table; }
__host__ __device__ constexpr int rows_max_waves(int bits, int mb, int amax, bool wide_table) {
    const int steps = bits == 4 ? 4 : 8;
    if (mb > 2 && (bits != 4 || amax != 4)) return 0;   // 33..64 rows: 4 bits, four row blocks side by side
    const int regs = amax * mb * 4 + steps * mb * 4 + (bits == 4 ? 84 : bits == 3 ? 116 : 108) + (wide_table ? 28 : 0)
                   + (bits == 4 && amax == 8 ? 20 : 0) + (rows_x_double(bits, mb, wide_table) ? steps * mb * 4 + 8 : 0);
    return regs <= 128 ? 16 : regs <= 168 ? 12 : regs <= 240 ? 8 : 0;
}

// RLUT: one table per output row (p.lut = [N, 2^bits]).  The tables of the pass's row blocks are built when the
// pass begins, sixteen copies per row block (the four lanes of a row share one; rowlut16_build), and slot a reads
// the copies of its own row block with the generic entry address.
template <int BITS, int GROUP, int MB, typename DT, int AMAX, bool RLUT = false>
__global__ __launch_bounds__(64 * (rows_max_waves(BITS, MB, AMAX, Tab<BITS, DT>::WIDE) > 0 ? rows_max_waves(BITS, MB, AMAX, Tab<BITS, DT>::WIDE) : 4))
void rows_kernel(const RowsParams p) {
    using Gm = Geo<BITS>;
    constexpr int TK = Gm::TK, STEPS = Gm::STEPS, TILE_BYTES = Gm::TILE_BYTES;
    constexpr int TPS = GROUP > TK ? GROUP / TK : 1;   // tiles that share one scale
    constexpr int NS = GROUP > TK ? 1 : TK / GROUP;    // scales per tile per row
    constexpr int SPG = GROUP / 32;                    // steps per group
    constexpr int LOG2C = perm_log2_copies<BITS, DT>();
    constexpr int LUT_BYTES = lut_row_table_bytes<BITS>();
    constexpr int D = 4;                               // steps whose table reads are in flight ahead of their use
    static_assert(STEPS % D == 0, "the ring of table reads runs on from one tile into the next");
    constexpr int NST = rows_tiles_in_flight(BITS, AMAX);   // weight tiles (and their scales) in flight per wave
    constexpr bool XDB = rows_x_double(BITS, MB, Tab<BITS, DT>::WIDE);
    // More than 32 rows: the activations come from a copy in operand order (fragment (kt, s, mb) = the 1 KiB the
    // wave's 64 lanes hold for K step s of tile kt and rows 16 mb .. 16 mb + 15, rows beyond M zero), written by
    // rows_xop_kernel just before this launch: every load is one contiguous KiB instead of sixteen rows' 64 bytes.
    constexpr bool XOP = MB > 2;
    static_assert(AMAX % NST == 0, "the row blocks of a pass are walked in rounds of the pipeline's stages");

    asm volatile("" ::"s"(p.X), "s"(p.packed), "s"(p.scales), "s"(p.lut), "s"(p.Y), "s"(p.packed_bytes), "s"(p.scale_bytes),
                 "s"(p.x_bytes), "s"(p.M), "s"(p.N), "s"(p.K), "s"(p.KT), "s"(p.SG2), "s"(p.SBL), "s"(p.tile_stride),
                 "s"(p.sblock_bytes), "s"(p.A), "s"(p.extra), "s"(p.NW), "s"(p.TQ), "s"(p.TR), "s"(p.RPR), "s"(p.lut_ltpe),
                 "s"(p.s_units), "s"(p.s_magic), "s"(p.SROW), "s"(p.red_off), "s"(p.tab_total), "s"(p.KS), "s"(p.TS), "s"(p.KSB), "s"(p.TQ1),
                 "s"(p.TR1));

    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15;                // row inside a 16-row block (A side) / activation row (B side)
    const int lo = lane >> 4;                // K octet
    char* lut = smem;
    char* sc = smem + (RLUT ? p.tab_total : LUT_BYTES);
    char* red = smem + p.red_off;
    constexpr bool PERM = !RLUT;             // the one-instruction entry address needs 256-byte entries
    constexpr int TB16 = rowlut16_bytes<BITS, DT>();

    LutSeed lut_seed{};
    if constexpr (!RLUT) lut_seed = lut_fetch<BITS>(p.lut, tid, p.lut_ltpe);
    __builtin_amdgcn_sched_barrier(0);
    const LutAddr la = make_lut_addr<BITS, DT>(lut, RLUT ? 4 : LOG2C, lane);
    // table of slot a (RLUT): the pass's row block a - skip; an empty slot reads the first one's
    auto la_of = [&](int a, int skip) {
        LutAddr r = la;
        if constexpr (RLUT) r.lane_base += (uint32_t)(a > skip ? a - skip : 0) * (uint32_t)TB16;
        return r;
    };
    const rsrc_t rW = make_rsrc(p.packed, p.packed_bytes);
    const rsrc_t rS = make_rsrc(p.scales, p.scale_bytes);
    const rsrc_t rX = make_rsrc(p.X, p.x_bytes);

    // this workgroup's row blocks and this wave's K tiles
    int share = (int)blockIdx.x, slice = 0;
    if (p.KS > 1) {
        share = (int)blockIdx.x / p.KS;
        slice = (int)blockIdx.x - share * p.KS;
    }
    const bool big = share < p.extra;
    const int nrb = p.A + (big ? 1 : 0);
    const int rb_first = share * p.A + (share < p.extra ? share : p.extra);
    // the slice's tiles (the first KSB slices have TS + 1) over the waves: tq each, the first trm waves one more
    const bool long_slice = slice < p.KSB;
    const int tq = long_slice ? p.TQ1 : p.TQ, trm = long_slice ? p.TR1 : p.TR;
    const int ka = slice * p.TS + (long_slice ? slice : p.KSB) + wave * tq + (wave < trm ? wave : trm);
    const int kb = ka + tq + (wave < trm ? 1 : 0);

    // activation rows m >= M lie beyond the X buffer and read as zero
    uint32_t xlane[MB];
    bool valid[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = li + 16 * mb;
        valid[mb] = m < p.M;
        xlane[mb] = XOP ? (uint32_t)mb * 1024u + 16u * (uint32_t)lane : ((uint32_t)m * (uint32_t)p.K + 8u * (uint32_t)lo) * 2u;
    }
    const uint32_t wlane = 16u * lane;
    (void)wlane;
    const uint32_t slane = (uint32_t)li * (uint32_t)p.SROW;

    struct Stage {
        WFrag<BITS> w;
        ScaleWords<NS> s;
    };
    // Slot (kt, a) of pass p0, a = 0 .. AMAX - 1: weight tile and scales of row block rb_first + p0 + a - skip,
    // where skip = AMAX - (row blocks of the pass): a short pass leaves its first slots empty.  Every slot
    // issues the same loads, in range or not (out of range: zeros, no memory traffic), and no load sits
    // under a branch: the waits on the load counter then name exactly the tile they need and leave the
    // younger ones in flight.
    auto load_w = [&](Stage& st, int p0, int skip, int kt, int a) {
        const bool in = a >= skip && kt < kb;
        const int rb = rb_first + p0 + a - skip;
        const uint32_t tw = (uint32_t)(rb >> p.SBL) * p.sblock_bytes + (uint32_t)(rb & ((1 << p.SBL) - 1)) * TILE_BYTES
                          + (uint32_t)kt * p.tile_stride;
        load_wfrag<BITS>(st.w, rW, in ? tw : kOutOfRange, lane);
    };
    // the slot's scales, from the pass's copy in LDS (an empty slot reads the first row's)
    auto load_s = [&](Stage& st, int skip, int kt, int a) {
        const bool in = a >= skip && kt < kb;
        const uint32_t ts = (uint32_t)(a - skip) * 16u * (uint32_t)p.SROW + slane + (uint32_t)(kt / TPS) * (NS * 2);
        lds_load_scales<NS>(st.s, sc + (in ? ts : 0u));
    };
    auto load_slot = [&](Stage& st, int p0, int skip, int kt, int a) {
        load_w(st, p0, skip, kt, a);
        load_s(st, skip, kt, a);
    };

    bool lut_ready = false;
    for (int p0 = 0; p0 < nrb; p0 += AMAX) {
        const int na = nrb - p0 < AMAX ? nrb - p0 : AMAX;      // row blocks of this pass
        const int skip = AMAX - na;                             // empty slots at the head of every K tile
        f32x4 acc[AMAX][MB];
#pragma unroll
        for (int a = 0; a < AMAX; ++a)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) acc[a][mb] = f32x4{0.f, 0.f, 0.f, 0.f};

        Stage st[NST];
#pragma unroll
        for (int a = 0; a < NST; ++a) {
            load_w(st[a], p0, skip, ka, a);
            __builtin_amdgcn_sched_barrier(0);
        }
        // Activations of two K tiles: the one being multiplied and the next one, asked for a whole tile ahead.  (A
        // load covers sixteen rows 2K bytes apart -- sixteen requests to one L2 channel -- and takes its time.)
        u32x4 bx[XDB ? 2 : 1][STEPS][MB];
        auto load_x_step = [&](auto buf, int kt, int s) {
            const uint32_t tx = kt < kb ? (uint32_t)kt * (XOP ? STEPS * MB * 1024 : TK * 2) : kOutOfRange;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                bx[decltype(buf)::value][s][mb] =
                    __builtin_amdgcn_raw_buffer_load_b128(rX, tx + xlane[mb] + (XOP ? MB * 1024u : 64u) * s, 0, kAuxNone);
        };
        auto load_x = [&](auto buf, int kt) {
#pragma unroll
            for (int s = 0; s < STEPS; ++s) load_x_step(buf, kt, s);
        };
        load_x(std::integral_constant<int, 0>{}, ka);
        __builtin_amdgcn_sched_barrier(0);
        {
            // The pass's scales: rows (rb_first + p0) * 16 onwards, na * 16 rows of SG2 bytes, one contiguous
            // range.  (Every wave is past the previous pass's K loop: its reduction began with a barrier.)
            // (s_units = 0: rows that are not whole 16-byte units -- the range, a multiple of 32 bytes that starts on one,
            // is copied as it lies, SROW = SG2, no padding between the rows)
            const int units = p.s_units ? na * 16 * p.s_units : na * p.SG2;
            const uint32_t gbase = (uint32_t)(rb_first + p0) * 16u * (uint32_t)p.SG2;
            for (int i = tid; i < units; i += p.NW * 64) {
                const int row = p.s_units <= 1 ? i : (int)__umulhi((uint32_t)i, p.s_magic);
                const int col = i - row * p.s_units;
                const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rS, gbase + 16u * (uint32_t)i, 0, kAuxNone);
                char* dst = p.s_units ? sc + (size_t)row * p.SROW + 16 * col : sc + 16 * (size_t)i;
                *reinterpret_cast<u32x4*>(dst) = v;
            }
        }
        if constexpr (RLUT) {
            // the raw tables of the pass's rows (one contiguous range) are staged in an area of their own in front
            // of the reduction slots (those may still be read by a slower wave of the previous pass), and the
            // sixteen-copy tables are built from there (nobody reads tables after a pass's K loop, which every wave
            // has left: the reduction began with a barrier)
            const rsrc_t rT = make_rsrc(p.lut, (uint32_t)p.N * (uint32_t)((1 << BITS) * 2));
            char* stage = red - AMAX * rowlut16_stage_bytes<BITS>();
            const int words = na * (rowlut16_stage_bytes<BITS>() / 4);
            const uint32_t tbase = (uint32_t)(rb_first + p0) * (uint32_t)rowlut16_stage_bytes<BITS>();
            for (int i = tid; i < words; i += p.NW * 64)
                *reinterpret_cast<uint32_t*>(stage + 4 * i) = __builtin_amdgcn_raw_buffer_load_b32(rT, tbase + 4u * (uint32_t)i, 0, kAuxNone);
            __syncthreads();
            rowlut16_build<BITS, DT>(lut, stage, na, tid, p.NW * 64);
        } else if (!lut_ready) {
            // the table is built while the first tiles are in flight (its own reads were issued before them)
            LutSeed seed = lut_seed;
            asm volatile("" : "+v"(seed.w[0]), "+v"(seed.w[1]), "+v"(seed.w[2]), "+v"(seed.w[3]));
            lut_build<BITS, DT>(lut, seed, (int)(reinterpret_cast<uintptr_t>(p.lut) >> 1) & 1, LOG2C, tid, p.lut_ltpe);
            lut_ready = true;
        }
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int a = 0; a < NST; ++a) load_s(st[a], skip, ka, a);
        __builtin_amdgcn_sched_barrier(0);

        // The table reads run D steps ahead of their use, across slots: when a slot begins, those of its
        // first D steps are already under way (issued by the slot before it, or here for the first).
        Raw<BITS, DT> raw[D];
#pragma unroll
        for (int s = 0; s < D; ++s) raw[s] = lookup_step<BITS, DT, PERM>(st[0].w, s, la_of(0, skip));
        __builtin_amdgcn_sched_barrier(0);

        // One K tile: buf = which set of bx holds its activations.  With two sets a tile beyond the wave's range
        // (the second of a pair when the wave owns an odd number) issues the same loads, out of range, and
        // multiplies nothing.  With one set the tile's last slot always multiplies (an empty pass slot there would
        // be a row block of zeros: the pass's empty slots are its first ones), because the next tile's activations
        // are fetched inside it, step by step as this tile's have had their last use.
        auto tile = [&](auto buf, int kt) {
            constexpr int B = decltype(buf)::value;
            if constexpr (XDB) {
                load_x(std::integral_constant<int, B ^ 1>{}, kt + 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            const bool live = !XDB || kt < kb;
#pragma unroll
            for (int a = 0; a < AMAX; ++a) {
                Stage& cur = st[a % NST];
                const Stage& nxt = st[(a + 1) % NST];
                const LutAddr la_cur = la_of(a, skip), la_nxt = la_of((a + 1) % AMAX, skip);
                if ((!XDB && a == AMAX - 1) || (live && a >= skip)) {
                    // dequantise the tile step by step and multiply it into row block a's accumulators
                    u32x4 aop[2];
#pragma unroll
                    for (int s = 0; s <= STEPS; ++s) {
                        if (s < STEPS) {
                            const ScaleReg<DT> sc = scale_of<DT, NS>(cur.s, s / SPG);
                            aop[s & 1] = scale4<BITS, DT>(raw[s % D], sc);
                            __builtin_amdgcn_sched_barrier(0);
                            raw[s % D] = s + D < STEPS ? lookup_step<BITS, DT, PERM>(cur.w, s + D, la_cur)
                                                       : lookup_step<BITS, DT, PERM>(nxt.w, s + D - STEPS, la_nxt);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        if (s > 0) {
#pragma unroll
                            for (int mb = 0; mb < MB; ++mb)
                                acc[a][mb] = mfma16x16x32<DT>(aop[(s - 1) & 1], bx[B][s - 1][mb], acc[a][mb]);
                            __builtin_amdgcn_sched_barrier(0);
                            if constexpr (!XDB) {
                                if (a == AMAX - 1) {
                                    load_x_step(std::integral_constant<int, 0>{}, kt + 1, s - 1);
                                    __builtin_amdgcn_sched_barrier(0);
                                }
                            }
                        }
                    }
                } else {
                    // an empty slot: only the next slot's first table reads
#pragma unroll
                    for (int s = 0; s < D; ++s) raw[s] = lookup_step<BITS, DT, PERM>(nxt.w, s, la_nxt);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // the slot NST ahead: further along this K tile, or among the first ones of the next
                const bool here = a + NST < AMAX;
                load_slot(cur, p0, skip, here ? kt : kt + 1, here ? a + NST : a + NST - AMAX);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        if constexpr (XDB) {
            for (int kt = ka; kt < kb; kt += 2) {
                tile(std::integral_constant<int, 0>{}, kt);
                tile(std::integral_constant<int, 1>{}, kt + 1);
            }
        } else {
            for (int kt = ka; kt < kb; ++kt) tile(std::integral_constant<int, 0>{}, kt);
        }

        // ---- add the waves' sums in wave order, RPR row blocks per round, and store ----
        for (int a0 = 0; a0 < na; a0 += p.RPR) {   // a0: first row block (of the pass) of this round
            __syncthreads();                       // the previous round's readers are done
#pragma unroll
            for (int a = 0; a < AMAX; ++a) {
                const int rbp = a - skip;          // slot a holds row block rbp of the pass
                if (rbp >= a0 && rbp < a0 + p.RPR) {
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        *reinterpret_cast<f32x4*>(red + ((size_t)(((rbp - a0) * MB + mb) * p.NW + wave) * 64 + lane) * 16) = acc[a][mb];
                }
            }
            __syncthreads();
            const int nr = na - a0 < p.RPR ? na - a0 : p.RPR;
            for (int task = wave; task < nr * MB; task += p.NW) {       // task = (row block of the round, M half); one wave each
                const int al = task / MB, mb = task - al * MB;
                f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
                const char* src = red + ((size_t)(task * p.NW) * 64 + lane) * 16;
#pragma unroll 4
                for (int w = 0; w < p.NW; ++w) sum += *reinterpret_cast<const f32x4*>(src + (size_t)w * 1024);
                if (p.KS > 1) {
                    // this workgroup's sums over its K slice go to its slot (output tile = row block of the share x block
                    // of sixteen rows of M; one pass: p0 = 0); nobody waits for the stores here
                    const int tile = (a0 + al) * MB + mb;
                    float* slot = p.slots + ((size_t)blockIdx.x * (AMAX * MB) + tile) * 256 + lane;
#pragma unroll
                    for (int i = 0; i < 4; ++i) __hip_atomic_store(slot + i * 64, sum[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    continue;
                }
                const int m = li + 16 * mb;
                if (m < p.M) {
                    const int n = (rb_first + p0 + a0 + al) * 16 + 4 * lo;
                    *reinterpret_cast<u32x2*>(p.Y + (size_t)m * p.N + n) = pack4<DT>(sum);
                }
            }
        }
        if (p.KS > 1) {
            // One arrival per workgroup, once all its stores are acknowledged; whichever of the share's KS workgroups
            // arrives last adds the slots of all of them in slice order, its own included, and writes Y.
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            uint32_t* counter = p.counters + (size_t)share * 16;               // one 64-byte line per share
            uint32_t* flag = reinterpret_cast<uint32_t*>(red);
            if (tid == 0) *flag = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            const uint32_t old = *flag;
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            if (old != (uint32_t)(p.KS - 1)) return;
            if (tid == 0) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            for (int tile = wave; tile < na * MB; tile += p.NW) {
                const int al = tile / MB, mb = tile - al * MB;
                f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
                const float* src = p.slots + ((size_t)(share * p.KS) * (AMAX * MB) + tile) * 256 + lane;
                for (int s0 = 0; s0 < p.KS; s0 += 4) {
                    // four slices' loads in flight together; a slice beyond the last reads the last one's and adds nothing
                    f32x4 v[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int s = s0 + j < p.KS ? s0 + j : p.KS - 1;
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            v[j][i] = __hip_atomic_load(src + (size_t)s * (AMAX * MB * 256) + i * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (s0 + j < p.KS) sum += v[j];
                }
                const int m = li + 16 * mb;
                if (m < p.M) {
                    const int n = (rb_first + al) * 16 + 4 * lo;
                    *reinterpret_cast<u32x2*>(p.Y + (size_t)m * p.N + n) = pack4<DT>(sum);
                }
            }
        }
        (void)valid;
    }
}

// The operand-order copy of X for rows_kernel's instances beyond 32 rows (the kernel sits beside the C ABI).  One workgroup per K tile; thread
// (row m, 16-byte chunk c of the tile's row) reads X[m, kt * TK + 8 c .. + 7] (zero for m >= M) and stores it where
// lane 16 (c mod 4) + m mod 16 of fragment (kt, c / 4, m / 16) expects it.
struct XopParams {
    const uint16_t* X;        // [M, K]
    uint16_t* Xop;            // KT x STEPS x MB x 1 KiB
    int M, K, MB, STEPS;      // STEPS = TK / 32
};

}  // namespace lutq
