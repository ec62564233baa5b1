// The fused kernel: stream packed weights HBM -> registers, dequantise through the LDS table,
// scale, multiply on the matrix cores, reduce partial sums across wavefronts and workgroups.
//
// Follows Algorithm 1 / Algorithm 2 of the paper in what is computed; the data path is
// re-designed for gfx950:
//   * weights never pass through LDS: the offline layout makes a wavefront's 128-bit global loads
//     land directly in A-operand order of v_mfma_f32_16x16x32 (weights on the A side, Y^T = W^ X^T);
//   * the only LDS resident is the vectorised table (Section 3.2), one private copy per bank column;
//   * M < 16 (or < 32) is padded with zero B-operand lanes in registers (the paper pads in shared
//     memory, "Limitations"), which costs no memory traffic;
//   * a workgroup is RS teams of KS wavefronts.  Team j works on row group RS*s + j of the
//     workgroup's current super-group s (a row group is R 16-row blocks streamed together by every
//     wave of the team, which share the activation fragments); the KS waves of a team split the K
//     range and are reduced through LDS.  With RS * R * (number of workgroups) = N / 16 every compute
//     unit streams the same number of bytes and no partial sum ever leaves the workgroup;
//   * otherwise work is split Stream-K style (Section 3.3): the (super-group x K tile) iteration
//     space is cut into `grid` contiguous ranges, so a workgroup's range may start and end in the
//     middle of an output tile.  Partial sums go to a global scratch slot per (workgroup, end, team);
//     an arrival counter per row group elects the last contributor, which adds the slots in a fixed
//     order (bit-reproducible results), writes Y and resets the counter.  Nobody ever waits on
//     another workgroup, so the kernel cannot deadlock whatever the number of resident workgroups.
#pragma once

#include <type_traits>

#include "lutq_device.hpp"

namespace lutq {

struct MatmulParams {
    const uint16_t* X;        // [M, K]
    const uint8_t* packed;
    const uint16_t* scales;   // [N, SG]
    const uint16_t* lut;
    uint16_t* Y;              // [M, N]
    uint32_t* counters;       // [NRG], zero on entry, zero on exit
    float* slots;             // [G][2][RS][accumulator registers per lane x 64 lanes]
    uint32_t packed_bytes;
    int M, N, K;
    int KT;                   // K tiles per row block
    int NRG;                  // row groups (N / (16 R)), a multiple of RS
    int G;                    // workgroups
    int TQ, TR;               // (NRG / RS) * KT = TQ * G + TR: workgroup b owns TQ (+1 if b < TR) iterations
    int SG;                   // scales per row (K / group)
    int SBL;                  // log2 of the row blocks per super-block of the packed layout (R divides it)
    int NW, KS, RS;           // waves per workgroup = KS waves per team x RS teams
    uint32_t kt_magic;        // floor(2^32 / KT) and floor(2^32 / KS): division by multiply-high, see div_magic
    uint32_t ks_magic;
    int lut_ltpe;             // log2 of the threads that build one table row together
    int xbuf_off;             // LDS byte offset of the shared activation buffers (XSH instances)
    int fast_reduce;          // the partial sums of all non-leading waves fit in the table area
    unsigned long long* trace;   // TRACE instances only: [G][kTraceWaves][kTraceStamps] device timestamps (else unused)
};

// Phase timestamps of the TRACE instances (measurement builds of a few instances, launched only by
// lutq_calib_matmul_trace): the constant 100 MHz device clock, read by every wave at these points of
// its first segment.
constexpr int kTraceWaves = 16;        // slots per workgroup (a workgroup has at most 16 waves)
enum TraceStamp {
    kTraceStart = 0,       // first instruction of the wave
    kTraceArgs = 1,        // kernel arguments have arrived in scalar registers
    kTraceIssued = 2,      // addresses computed, table values requested, first tiles requested
    kTraceTable = 3,       // table built, workgroup barrier passed
    kTraceFirstTile = 4,   // first tile of weights has arrived and is multiplied
    kTraceLoopDone = 5,    // K loop finished
    kTraceReduced = 6,     // waves of the team reduced through LDS
    kTraceEnd = 7,         // outputs stored (or partial sums handed over)
    kTraceStamps = 8
};

// A partial-sum slot holds one wave's accumulators: R row blocks x MB halves of M x 4 registers x 64 lanes.
__host__ __device__ constexpr int slot_floats(int r, int mb) { return r * mb * 4 * 64; }
// the largest one: R = 4, M > 16
constexpr int kSlotFloats = slot_floats(4, 2);

// n / d for 0 <= n < 2^31 with m = floor(2^32 / d) (0xffffffff for d = 1) computed on the host: the
// multiply-high is the quotient or one less, so one correction step makes it exact.  A run-time
// integer division costs some thirty instructions here, and the prologue runs in every wave.
__device__ __forceinline__ int div_magic(int n, uint32_t m, int d) {
    int q = (int)__umulhi((uint32_t)n, m);
    if (n - q * d >= d) ++q;
    return q;
}

// The (NRG / RS) * KT iterations (super-group major) are cut into G contiguous ranges; the first TR
// ranges hold TQ + 1 iterations, the others TQ.  All of it fits 32 bits (checked on the host).
__device__ __forceinline__ int range_begin(int g, int tq, int tr) { return g * tq + (g < tr ? g : tr); }
__device__ __forceinline__ int owner_of(int t, int tq, int tr) {
    const int big = tr * (tq + 1);
    return t < big ? t / (tq + 1) : tr + (t - big) / tq;
}

// LDS bytes of one launch (host and device agree through these functions):
// [table, 256-byte entry stride][one partial-sum slot per team][one 1 KiB scale-chunk area per wave]
__host__ __device__ constexpr int red_bytes(int nreg, int rs) { return nreg * 256 * rs; }
// Activation pieces: one piece is the B operand of one (K step, 16-row half of M) = 64 lanes x 16 bytes.
constexpr int kXPiecesPerWave = 2;       // most pieces of a tile that one wave stages (shared-activation instances)
template <int BITS>
__host__ __device__ constexpr int x_pieces(int mb) { return Geo<BITS>::STEPS * mb; }
// offset of the shared activation buffers = end of the other areas
template <int BITS>
__host__ __device__ constexpr int matmul_xbuf_offset(int r, int mb, int nw, int rs, bool sch) {
    return lut_row_table_bytes<BITS>() + red_bytes(r * mb * 4, rs) + (sch ? nw * 1024 : 0);
}
// [..][shared-activation instances: 2 (double buffer) x KS (K parts) x pieces x 1 KiB]
template <int BITS>
__host__ __device__ constexpr int matmul_lds_bytes(int r, int mb, int nw, int rs, bool sch, bool xsh) {
    return matmul_xbuf_offset<BITS>(r, mb, nw, rs, sch) + (xsh ? 2 * (nw / rs) * x_pieces<BITS>(mb) * 1024 : 0);
}

// Rough count of the registers live in the K loop (tiles in flight, accumulators, lookup ring,
// addresses): decides which instances can be held to 128 registers, i.e. four waves per SIMD.
template <int BITS>
__host__ __device__ constexpr int matmul_reg_estimate(int r, int mb, int p, int xm, bool wide_table, int xsh) {
    const int wregs = BITS == 3 ? 6 : 4;
    const int xl = Geo<BITS>::STEPS * xm / 16;
    const int na = xm == 16 ? mb : 16 / xm;               // accumulators per row block
    // activations in flight per tile: the wave's own fragments, or its share of the staged pieces
    // (plus two steps' worth of operands read back from LDS)
    const int xregs = xsh ? xsh * 4 : xl * mb * 4;
    return p * (r * wregs + xregs + 4) + (xsh ? 2 * mb * 4 : 0) + r * na * 4 + 46 + (wide_table ? 12 : 0);
}
template <int BITS>
__host__ __device__ constexpr bool matmul_wide_fits(int r, int mb, int p, int xm, bool wide_table, int xsh) {
    return matmul_reg_estimate<BITS>(r, mb, p, xm, wide_table, xsh) <= 124;
}

// Template parameters: bit width, group size, MB = 16-row halves of M (1: M <= 16, 2: M <= 32),
// R = 16-row weight blocks a wave streams together, P = tiles in flight per wave, SCH = scales are
// fetched as 16-byte chunks per row (needs K/group % 8 == 0) and handed to the lanes through LDS
// instead of being loaded per tile.
// XM = activation rows that one 16-lane row of the B operand is loaded for: 16 is the plain layout
// (lane i holds row i; one 128-bit load per 32-wide K step).  XM = 4 (M <= 4 only) packs four K steps
// into one load: lane i holds row i % 4 of step i / 4.  The matrix instruction of step s then gets the
// right activations in columns 4 (s % 4) .. 4 (s % 4) + 3 only, so each of the four step positions
// accumulates into its own registers (the other twelve columns multiply activations of other steps
// and are never read), and the four accumulators are folded together, with three row rotations, once
// per output tile.  This cuts the registers that hold activations in flight to a quarter and issues a
// quarter of the activation loads.  XM = 8 (M <= 8) is the same with two K steps per load: lane i
// holds row i % 8 of step i / 8, two accumulators per row block, one rotation.
// WIDE: the instance is compiled for up to 16 waves per workgroup and therefore at most 128
// registers (four waves per SIMD, or two 8-wave workgroups with their two 64 KiB tables in the
// 160 KiB of LDS); otherwise for up to 8 waves and as many registers as it likes.
// XSH (plain layout, M > 4): the activations go through LDS and are shared by the teams.  All teams
// of a workgroup walk the same K tiles, so without sharing each of them fetches the same M x TK
// activations per tile, which for M = 16..32 is one to two times the weight bytes through the
// 64 B/clk vector memory path.  With XSH the waves that work on the same K part (one per team) split
// the tile's pieces between them (at most two each), store them in LDS in operand order one tile
// ahead, double buffered, and every wave reads its B operands from there; one workgroup barrier per
// tile keeps writers and readers apart, and every wave runs the same number of rounds.
// The number of waves and their arrangement in teams are run-time values.
template <int BITS, int GROUP, int MB, int R, typename DT, int P, bool SCH, int XM, bool WIDE, int XPIECES, bool RLUT = false,
          bool TRACE = false>
__global__ __launch_bounds__(WIDE ? 1024 : 512) void matmul_kernel(const MatmulParams p) {
    static_assert(XM == 16 || ((XM == 4 || XM == 8) && MB == 1), "packed activation loads exist for M <= 8 only");
    constexpr bool XSH = XPIECES != 0;       // activations shared through LDS; XPIECES = pieces one wave stages (1 or 2)
    static_assert(XPIECES >= 0 && XPIECES <= kXPiecesPerWave, "a wave stages one or two pieces");
    static_assert(!XSH || XM == 16, "activations are shared through LDS in the plain layout only");
    static_assert(!RLUT || (R == 1 && !XSH), "one table per output row: one row block per workgroup at a time");
    using Gm = Geo<BITS>;
    constexpr int TK = Gm::TK, STEPS = Gm::STEPS, TILE_BYTES = Gm::TILE_BYTES;
    constexpr int TPS = GROUP > TK ? GROUP / TK : 1;   // tiles that share one scale (a group longer than a tile)
    constexpr int NS = GROUP > TK ? 1 : TK / GROUP;    // scales per tile per row
    constexpr int SPG = GROUP / 32;          // steps per group
    constexpr int NREG = R * MB * 4;         // accumulator registers per lane
    constexpr int TPC = 8 * TPS / NS;        // tiles covered by one 16-byte scale chunk
    constexpr int LOG2C = perm_log2_copies<BITS, DT>();
    constexpr int LUT_BYTES = lut_lds_bytes<BITS, DT>(LOG2C);
    static_assert(LUT_BYTES == lut_row_table_bytes<BITS>(), "one 256-byte row per entry");
    constexpr int U = STEPS * R;             // (step, row block) items of one tile
    constexpr int D = U < 4 ? U : 4;         // table reads kept in flight ahead of their use
    constexpr int XS = 16 / XM;              // K steps covered by one activation load
    constexpr int XL = STEPS / XS;           // activation loads per tile (per 16-row half of M)
    constexpr int NA = XM == 16 ? MB : XS;   // accumulators per row block: M halves, or step positions
    constexpr int NP = STEPS * MB;           // activation pieces (K step, M half) of one tile, 1 KiB each
    constexpr int XPW = XSH ? XPIECES : 1;   // pieces one wave stages (RS * XPW >= NP is checked on the host)
    constexpr int NX = XSH ? XPW : XL;       // activation loads per tile held in a stage
    constexpr int NXM = XSH ? 1 : MB;

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
    // Every scalar of the parameter block is used in the entry block, so that the argument segment
    // is fetched with one round trip instead of one per basic block that first needs a field.
    asm volatile("" ::"s"(p.X), "s"(p.packed), "s"(p.scales), "s"(p.lut), "s"(p.Y), "s"(p.counters), "s"(p.slots));
    asm volatile("" ::"s"(p.packed_bytes), "s"(p.M), "s"(p.N), "s"(p.K), "s"(p.KT), "s"(p.NRG), "s"(p.G), "s"(p.TQ),
                 "s"(p.TR), "s"(p.SG), "s"(p.SBL), "s"(p.NW), "s"(p.KS), "s"(p.RS), "s"(p.fast_reduce),
                 "s"(p.kt_magic), "s"(p.ks_magic), "s"(p.lut_ltpe), "s"(p.xbuf_off));
    stamp(kTraceArgs);

    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int team = div_magic(wave, p.ks_magic, p.KS);   // which row group of the super-group
    const int kpart = wave - team * p.KS;    // which part of the K range
    const int li = lane & 15;                // row inside a 16-row block (A side) / activation row (B side)
    const int lo = lane >> 4;                // K octet

    char* lut = smem;
    float* red = reinterpret_cast<float*>(smem + LUT_BYTES) + team * (NREG * 64);   // this team's slot
    char* sc_lds = smem + LUT_BYTES + red_bytes(NREG, p.RS) + wave * 1024;         // this wave's 64 rows x 16 B

    // issued before any weight load (see below); with one table per row the table is fetched per row block
    LutSeed lut_seed{};
    if constexpr (!RLUT) lut_seed = lut_fetch<BITS>(p.lut, tid, p.lut_ltpe);
    __builtin_amdgcn_sched_barrier(0);
    const LutAddr la = make_lut_addr<BITS, DT>(lut, LOG2C, lane);
    bool lut_ready = false;

    const rsrc_t rW = make_rsrc(p.packed, p.packed_bytes);
    const rsrc_t rS = make_rsrc(p.scales, (uint32_t)p.N * (uint32_t)p.SG * 2u);
    const rsrc_t rX = make_rsrc(p.X, (uint32_t)p.M * (uint32_t)p.K * 2u);

    // activation rows m >= M fall outside the X buffer and read as zero: the padding of the
    // matrix instruction's 16 (or 32) columns costs no memory traffic
    bool valid[MB];
    uint32_t xlane[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = li + 16 * mb;
        valid[mb] = m < p.M;
        // packed form: row li % XM, K step li / XM of the load's group of XS steps
        xlane[mb] = ((uint32_t)(XM == 16 ? m : li % XM) * (uint32_t)p.K + 32u * (uint32_t)(XM == 16 ? 0 : li / XM)
                     + 8u * lo) * 2u;
    }
    // shared activations: the pieces this wave stages (team, team + RS, ...), where they come from
    // and where they go in a buffer; the buffer of K part `kpart` and parity b starts at
    // xbuf + (b * KS + kpart) * NP KiB
    char* xbuf = smem + p.xbuf_off;
    bool xp_ok[XPW];
    uint32_t xp_src[XPW], xp_dst[XPW];
#pragma unroll
    for (int i = 0; i < XPW; ++i) {
        const int pi = team + p.RS * i;                       // piece = step * MB + M half
        xp_ok[i] = XSH && pi < NP;
        const int m = li + 16 * (pi % MB);
        xp_src[i] = ((uint32_t)m * (uint32_t)p.K + 32u * (uint32_t)(pi / MB) + 8u * lo) * 2u;
        xp_dst[i] = ((uint32_t)(kpart * NP + pi) * 64u + (uint32_t)lane) * 16u;
    }
    const uint32_t xpar_bytes = (uint32_t)(p.KS * NP) * 1024u;       // one parity's buffers
    const uint32_t tile_stride = (uint32_t)TILE_BYTES << p.SBL;        // bytes from K tile kt to kt+1
    const uint32_t sblock_bytes = (uint32_t)p.KT * tile_stride;         // packed bytes of one super-block
    const uint32_t srow_bytes = 16u * (uint32_t)p.SG * 2u;             // scale bytes of one 16-row block

    int t0 = range_begin((int)blockIdx.x, p.TQ, p.TR);
    const int t1 = t0 + p.TQ + ((int)blockIdx.x < p.TR ? 1 : 0);
    const int tbeg = t0;

    struct Stage {
        WFrag<BITS> w[R];
        ScaleWords<NS> s[SCH ? 1 : R];     // direct mode: this lane's scales of the tile, per row block
        u32x4 chunk;                       // chunk mode: 8 consecutive scales of row `lane` of the wave's rows
        u32x4 x[NX][NXM];                  // XSH: this wave's pieces of the *next* tile
    };

    while (t0 < t1) {
        const int sg = div_magic(t0, p.kt_magic, p.KT); // super-group
        const int ka = t0 - sg * p.KT;
        const int rem = (t1 - t0 < p.KT - ka) ? (t1 - t0) : (p.KT - ka);
        const int kb = ka + rem;
        const int rg = sg * p.RS + team;                // this team's row group
        const int wa = ka + div_magic(kpart * rem, p.ks_magic, p.KS);
        const int wb = ka + div_magic((kpart + 1) * rem, p.ks_magic, p.KS);
        const bool last_segment = (t0 + rem == t1);

        f32x4 acc[R][NA];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int a = 0; a < NA; ++a) acc[r][a] = f32x4{0.f, 0.f, 0.f, 0.f};

        const int rb0 = rg * R;                                                          // first row block
        const uint32_t wrow = (uint32_t)(rb0 >> p.SBL) * sblock_bytes + (uint32_t)(rb0 & ((1 << p.SBL) - 1)) * TILE_BYTES;
        const uint32_t slane = (uint32_t)rb0 * srow_bytes + (uint32_t)li * p.SG * 2u;    // direct mode
        const uint32_t clane = lane < 16 * R ? (uint32_t)rb0 * srow_bytes + (uint32_t)lane * p.SG * 2u
                                             : kOutOfRange;                              // chunk mode

        // Loads of tile kt; kt >= wb turns every offset out of range (zeros, no traffic).
        // (`prologue`: the loads that fill the pipeline before the table is built.  There the scale-chunk
        // load is issued unconditionally, so that the number of loads between the table fetch and the
        // wait for it is the same on every path and the wait counts exactly the table's two loads
        // instead of, conservatively, the first tile as well.)
        auto load_stage = [&](Stage& st, int kt, auto prologue) {
            const bool in = kt < wb;
            const uint32_t tw = in ? wrow + (uint32_t)kt * tile_stride : kOutOfRange;
            const uint32_t tx = in ? (uint32_t)kt * (TK * 2) : kOutOfRange;
#pragma unroll
            for (int r = 0; r < R; ++r) load_wfrag<BITS>(st.w[r], rW, tw + r * TILE_BYTES, lane);
            if constexpr (SCH) {
                const bool first = in && ((kt % TPC) == 0 || kt == wa);
                const uint32_t tc = first ? (uint32_t)(kt / TPC) * 16u : kOutOfRange;
                // seven of eight chunk loads would be out of range: an out-of-range load still costs its
                // turn in the address unit (as much as the weight load itself), so they are branched
                // around (the condition is uniform over the wave).  The shared-activation instances keep
                // the unconditional form: there the extra control flow costs more than it saves.
                if constexpr (XSH) st.chunk = __builtin_amdgcn_raw_buffer_load_b128(rS, tc + clane, 0, kAuxNone);
                else if (decltype(prologue)::value || first) st.chunk = __builtin_amdgcn_raw_buffer_load_b128(rS, tc + clane, 0, kAuxNone);
            } else {
                const uint32_t ts = in ? (uint32_t)(kt / TPS) * (NS * 2) : kOutOfRange;
#pragma unroll
                for (int r = 0; r < R; ++r) load_scales<NS>(st.s[r], rS, ts + slane + r * srow_bytes);
            }
            if constexpr (XSH) {
                // pieces of tile kt + 1: they are stored to LDS while tile kt is computed
                const uint32_t tx1 = kt + 1 < wb ? (uint32_t)(kt + 1) * (TK * 2) : kOutOfRange;
#pragma unroll
                for (int i = 0; i < XPW; ++i)
                    st.x[i][0] = __builtin_amdgcn_raw_buffer_load_b128(rX, xp_ok[i] ? tx1 + xp_src[i] : kOutOfRange, 0, kAuxNone);
            } else {
#pragma unroll
                for (int j = 0; j < XL; ++j)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        st.x[j][mb] = __builtin_amdgcn_raw_buffer_load_b128(rX, tx + xlane[mb] + 64u * XS * j, 0, kAuxNone);
            }
        };
        // `round` counts the tiles of this segment (same in every wave of the workgroup); XSH only
        auto compute_stage = [&](const Stage& st, int kt, int round) {
            const char* bsrc = xbuf + (uint32_t)(round & 1) * xpar_bytes + ((uint32_t)(kpart * NP) * 64u + (uint32_t)lane) * 16u;
            if constexpr (XSH) {
                // next tile's pieces into the other buffer (its readers passed the last barrier)
                char* dst = xbuf + (uint32_t)((round + 1) & 1) * xpar_bytes;
#pragma unroll
                for (int i = 0; i < XPW; ++i)
                    if (xp_ok[i]) *reinterpret_cast<u32x4*>(dst + xp_dst[i]) = st.x[i][0];
                if (kt >= wb) return;                   // nothing of this wave's own left (the caller still syncs)
            }
            ScaleWords<NS> sw[R];
            if constexpr (SCH) {
                // a new chunk starts at this tile: every lane parks its row's 8 scales in LDS, then each
                // lane picks the scales of its own rows (LDS operations of one wave complete in order)
                if ((kt % TPC) == 0 || kt == wa) {
                    asm volatile("" ::: "memory");      // keep earlier reads of the old chunk before this store
                    *reinterpret_cast<u32x4*>(sc_lds + 16 * lane) = st.chunk;
                    asm volatile("" ::: "memory");      // and the reads below after it
                }
                const char* src = sc_lds + 16 * li + ((kt % TPC) / TPS) * (NS * 2);
#pragma unroll
                for (int r = 0; r < R; ++r) lds_load_scales<NS>(sw[r], src + 256 * r);
            } else {
#pragma unroll
                for (int r = 0; r < R; ++r) sw[r] = st.s[r];
            }
            // items u = (step s, row block r), r fastest; the table reads of item u + D are issued
            // before item u is scaled and multiplied
            // (scheduling barriers pin this order: left alone, the compiler sinks part of an item's
            // table reads to just before their use and every item then waits out the LDS latency)
            Raw<BITS, DT> raw[D];
#pragma unroll
            for (int u = 0; u < D; ++u) raw[u] = lookup_step<BITS, DT, true>(st.w[u % R], u / R, la);
            __builtin_amdgcn_sched_barrier(0);
            // the matrix instruction of item u is issued after the scaling of item u + 1, so that it
            // never has to wait for operands that were written by the instructions just before it
            u32x4 a[2];
            u32x4 bx[2][MB];                            // XSH: B operands of the current and the next step
            if constexpr (XSH) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) bx[0][mb] = *reinterpret_cast<const u32x4*>(bsrc + mb * 1024);
            }
#pragma unroll
            for (int u = 0; u <= U; ++u) {
                if (u < U) {
                    const int s = u / R, r = u % R;
                    const ScaleReg<DT> sc = scale_of<DT, NS>(sw[r], s / SPG);
                    a[u & 1] = scale4<BITS, DT>(raw[u % D], sc);
                    __builtin_amdgcn_sched_barrier(0);
                    if (u + D < U) {
                        raw[u % D] = lookup_step<BITS, DT, true>(st.w[(u + D) % R], (u + D) / R, la);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if (u > 0) {
                    const int s = (u - 1) / R, r = (u - 1) % R;
                    if constexpr (XSH) {
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb)
                            acc[r][mb] = mfma16x16x32<DT>(a[(u - 1) & 1], bx[s & 1][mb], acc[r][mb]);
                        // the operands of step s + 1 are fetched as soon as the last product of step
                        // s - 1 (which used the same registers) has been issued
                        if (r == 0 && s + 1 < STEPS) {
#pragma unroll
                            for (int mb = 0; mb < MB; ++mb)
                                bx[(s + 1) & 1][mb] = *reinterpret_cast<const u32x4*>(bsrc + ((s + 1) * MB + mb) * 1024);
                        }
                    } else if constexpr (XM == 16) {
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb)
                            acc[r][mb] = mfma16x16x32<DT>(a[(u - 1) & 1], st.x[s][mb], acc[r][mb]);
                    } else {
                        acc[r][s % XS] = mfma16x16x32<DT>(a[(u - 1) & 1], st.x[s / XS][0], acc[r][s % XS]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };

        // The scheduling barriers keep the loads of different stages in program order, so that the
        // wait before a stage's first use only has to cover that stage's own loads.
        RowTab rowtab{};
        if constexpr (RLUT) {
            // this lane's row of the new row block (one team: rg is the row block); issued before the
            // tile prefetch so that waiting for it does not wait for the tiles
            rowtab = rowlut_fetch<BITS>(p.lut, (int64_t)rg * 16 + li);
            __builtin_amdgcn_sched_barrier(0);
        }
        Stage st[P];
        u32x4 xfirst[XPW];                              // XSH: this wave's pieces of the segment's first tile
        if constexpr (XSH) {
            const uint32_t tx0 = wa < wb ? (uint32_t)wa * (TK * 2) : kOutOfRange;
#pragma unroll
            for (int i = 0; i < XPW; ++i)
                xfirst[i] = __builtin_amdgcn_raw_buffer_load_b128(rX, xp_ok[i] ? tx0 + xp_src[i] : kOutOfRange, 0, kAuxNone);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int q = 0; q < P; ++q) {
            load_stage(st[q], wa + q, std::true_type{});
            __builtin_amdgcn_sched_barrier(0);
        }
        stamp(kTraceIssued);
        if constexpr (RLUT) {
            // every wave has left the K loop of the previous row block (the reduction's barriers lie in
            // between), so the copies can be overwritten with this row block's tables
            asm volatile("" : "+v"(rowtab.a), "+v"(rowtab.b));
            rowlut_build<BITS, DT>(lut, rowtab, wave, p.NW, lane);
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
        } else if (!lut_ready) {
            // first segment: the table is built while the first tiles are in flight (its own reads
            // of T were issued before them, so waiting for T does not wait for the tiles)
            // (the empty statement keeps the wait for T, and the arithmetic on it, from being hoisted
            // out of the segment loop to a point before the prefetch)
            LutSeed seed = lut_seed;
            asm volatile("" : "+v"(seed.w[0]), "+v"(seed.w[1]), "+v"(seed.w[2]), "+v"(seed.w[3]));
            lut_build<BITS, DT>(lut, seed, (int)(reinterpret_cast<uintptr_t>(p.lut) >> 1) & 1, LOG2C, tid, p.lut_ltpe);
            if constexpr (!XSH) __syncthreads();
            lut_ready = true;
            __builtin_amdgcn_sched_barrier(0);
        }
        stamp(kTraceTable);
        if constexpr (XSH) {
            // first tile's pieces into buffer 0 (every reader of the previous segment has passed its
            // last barrier); the barrier also publishes the table
#pragma unroll
            for (int i = 0; i < XPW; ++i)
                if (xp_ok[i]) *reinterpret_cast<u32x4*>(xbuf + xp_dst[i]) = xfirst[i];
            __syncthreads();
            // every wave of the workgroup runs the same number of rounds (the longest K part's), one
            // barrier each, whether or not it still has tiles of its own
            const int rounds = div_magic(rem + p.KS - 1, p.ks_magic, p.KS);
            for (int it = 0; it < rounds; it += P) {
#pragma unroll
                for (int q = 0; q < P; ++q) {
                    compute_stage(st[q], wa + it + q, it + q);
                    __syncthreads();
                    __builtin_amdgcn_sched_barrier(0);
                    load_stage(st[q], wa + it + q + P, std::false_type{});
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        } else {
            // steady state while a further group of P tiles is left; the last tiles (they are already
            // in flight) are computed without issuing prefetches beyond the wave's range, which would
            // be out of range and return nothing but still take their turn in the address unit
            int kt = wa;
            for (; kt + P < wb; kt += P) {
#pragma unroll
                for (int q = 0; q < P; ++q) {
                    compute_stage(st[q], kt + q, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    stamp(kTraceFirstTile);
                    load_stage(st[q], kt + q + P, std::false_type{});
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int q = 0; q < P; ++q) {
                if (kt + q < wb) compute_stage(st[q], kt + q, 0);
                __builtin_amdgcn_sched_barrier(0);
                stamp(kTraceFirstTile);
            }
        }
        stamp(kTraceLoopDone);

        if constexpr (XM != 16) {
            // fold the step positions: columns 4 j .. 4 j + 3 of accumulator j move to columns 0 .. 3
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int j = 1; j < XS; ++j) {
                    const u32x4 t = rotate_rows(__builtin_bit_cast(u32x4, acc[r][j]), XM * j);
                    acc[r][0] += __builtin_bit_cast(f32x4, t);
                }
        }

        // ---- reduce the waves of each team through LDS, in wave order ----
        if (p.KS > 1) {
            if (p.fast_reduce && last_segment) {
                // nobody needs the table any more: every non-leading wave parks its sums there, the
                // team's leading wave adds them up
                __syncthreads();
                float* area = reinterpret_cast<float*>(lut);
                if (kpart != 0) {
                    float* dst = area + (size_t)(team * (p.KS - 1) + kpart - 1) * (NREG * 64) + lane;
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                            for (int i = 0; i < 4; ++i) dst[((r * MB + mb) * 4 + i) * 64] = acc[r][mb][i];
                }
                __syncthreads();
                if (kpart == 0) {
                    // (four partial sums per round: their LDS reads are in flight together)
#pragma unroll 4
                    for (int w = 0; w < p.KS - 1; ++w) {
                        const float* src = area + (size_t)(team * (p.KS - 1) + w) * (NREG * 64) + lane;
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                                for (int i = 0; i < 4; ++i) acc[r][mb][i] += src[((r * MB + mb) * 4 + i) * 64];
                    }
                }
            } else {
#pragma unroll 1
                for (int w = 1; w < p.KS; ++w) {
                    if (kpart == w) {
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                                for (int i = 0; i < 4; ++i) red[((r * MB + mb) * 4 + i) * 64 + lane] = acc[r][mb][i];
                    }
                    __syncthreads();
                    if (kpart == 0) {
#pragma unroll
                        for (int r = 0; r < R; ++r)
#pragma unroll
                            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                                for (int i = 0; i < 4; ++i) acc[r][mb][i] += red[((r * MB + mb) * 4 + i) * 64 + lane];
                    }
                    __syncthreads();
                }
            }
        }

        stamp(kTraceReduced);
        // ---- emit: whole output tile -> Y; otherwise the Stream-K fix-up ----
        // Partial sums and counters are moved with device-scope (agent) atomic loads/stores, which
        // bypass the per-XCD L2 for coherence.  No device-scope fence is used: on this multi-die part
        // such a fence writes back and invalidates the whole L2 and costs far more than the kernel.
        // Ordering comes from completion instead: the writer waits until its stores are acknowledged
        // before it bumps the counter, and the reader issues its loads only after the counter value
        // that proves it is last has come back.
        if (kpart == 0) {
            bool write_y = (ka == 0 && kb == p.KT);
            if (!write_y) {
                // (the split is re-read through an empty statement so that the divisions below stay on
                // this rarely taken path instead of being hoisted into every wave's prologue)
                int tq = p.TQ, tr = p.TR;
                asm volatile("" : "+s"(tq), "+s"(tr));
                const int tile0 = sg * p.KT;
                const int g_first = owner_of(tile0, tq, tr);
                const int g_last = owner_of(tile0 + p.KT - 1, tq, tr);
                const int which = (t0 == tbeg) ? 0 : 1;
                float* slot = p.slots + (((size_t)blockIdx.x * 2 + which) * p.RS + team) * slot_floats(R, MB) + lane;
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        if (valid[mb])
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                __hip_atomic_store(slot + ((r * MB + mb) * 4 + i) * 64, acc[r][mb][i],
                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // wait for the stores to complete
                __builtin_amdgcn_s_waitcnt(0);
                uint32_t old = 0;
                if (lane == 0)
                    old = __hip_atomic_fetch_add(p.counters + rg, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                old = __builtin_amdgcn_readfirstlane(old);
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                if (old == (uint32_t)(g_last - g_first)) {
                    // last contributor: add every slot in workgroup order (own one included)
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb) acc[r][mb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
                    for (int g = g_first; g <= g_last; ++g) {
                        const int gbeg = range_begin(g, tq, tr);
                        const int gw = (div_magic(gbeg, p.kt_magic, p.KT) == sg) ? 0 : 1;   // slot 0 iff sg is g's first super-group
                        const float* src = p.slots + (((size_t)g * 2 + gw) * p.RS + team) * slot_floats(R, MB) + lane;
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
    if constexpr (TRACE) {
        __builtin_amdgcn_s_waitcnt(0);                       // the stores of Y have been acknowledged
        stamp(kTraceEnd);
        if (p.trace && lane == 0) {
            unsigned long long* o = p.trace + ((size_t)blockIdx.x * kTraceWaves + wave) * kTraceStamps;
#pragma unroll
            for (int i = 0; i < kTraceStamps; ++i) o[i] = tr[i];
        }
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
    uint32_t packed_bytes;
    int N, K, KT, SG;
    int SB;           // row blocks per super-block of the packed layout
    int64_t tiles;    // (N/16) * KT
    int log2c;
};

template <int BITS, int GROUP, typename DT>
__global__ __launch_bounds__(256) void dequant_kernel(const DequantParams p) {
    using Gm = Geo<BITS>;
    constexpr int TK = Gm::TK, STEPS = Gm::STEPS, TILE_BYTES = Gm::TILE_BYTES;
    constexpr int TPS = GROUP > TK ? GROUP / TK : 1, NS = GROUP > TK ? 1 : TK / GROUP, SPG = GROUP / 32;
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    build_lut<BITS, DT>(smem, p.lut, p.log2c, tid, 256);
    const LutAddr la = make_lut_addr<BITS, DT>(smem, p.log2c, lane);
    __syncthreads();
    const int li = lane & 15, lo = lane >> 4;
    const rsrc_t rW = make_rsrc(p.packed, p.packed_bytes);
    const rsrc_t rS = make_rsrc(p.scales, (uint32_t)p.N * (uint32_t)p.SG * 2u);
    for (int64_t t = (int64_t)blockIdx.x * 4 + wave; t < p.tiles; t += (int64_t)gridDim.x * 4) {
        // t counts tiles in storage order: super-block, K tile, row block inside the super-block
        const int64_t per_sb = (int64_t)p.KT * p.SB;
        const int64_t sb = t / per_sb;
        const int in_sb = (int)(t - sb * per_sb);
        const int kt = in_sb / p.SB;
        const int64_t rb = sb * p.SB + in_sb % p.SB;
        WFrag<BITS> f;
        load_wfrag<BITS>(f, rW, (uint32_t)t * TILE_BYTES, lane);
        ScaleWords<NS> sw;
        load_scales<NS>(sw, rS, (((uint32_t)rb * 16 + li) * (uint32_t)p.SG + (uint32_t)(kt / TPS) * NS) * 2u);
        uint16_t* out = p.W + ((size_t)rb * 16 + li) * p.K + (size_t)kt * TK + 8 * lo;
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const ScaleReg<DT> sc = scale_of<DT, NS>(sw, s / SPG);
            const u32x4 a = scale4<BITS, DT>(lookup_step<BITS, DT, false>(f, s, la), sc);
            *reinterpret_cast<u32x4*>(out + 32 * s) = a;
        }
    }
}

}  // namespace lutq
