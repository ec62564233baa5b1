// Device-side building blocks shared by the fused matmul kernel and the dequantise
// kernel: tile geometry per bit width, the vectorised lookup table in LDS
// (Section 3.2 of the paper: a table over all index pairs, duplicated to avoid bank
// conflicts), bit-slice combination for 3-bit (Section 3.1), and group scaling.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lutq {

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct F16 {};
struct BF16 {};

// Tile geometry of the packed layout (see lutq_pack.cpp).
template <int BITS> struct Geo;
template <> struct Geo<4> {
    static constexpr int TK = 128, STEPS = 4, TILE_BYTES = 1024;
    static constexpr int ENTRIES = 256, ENTRY_BYTES = 4, MAX_LOG2_COPIES = 5;   // pair table
};
template <> struct Geo<3> {
    static constexpr int TK = 256, STEPS = 8, TILE_BYTES = 1536;
    static constexpr int ENTRIES = 64, ENTRY_BYTES = 4, MAX_LOG2_COPIES = 5;    // pair table, 6-bit address
};
template <> struct Geo<2> {
    static constexpr int TK = 256, STEPS = 8, TILE_BYTES = 1024;
    static constexpr int ENTRIES = 256, ENTRY_BYTES = 8, MAX_LOG2_COPIES = 4;   // quad table
};

// What one table entry holds.  fp16: the two (pair table) or four (quad table) 16-bit values.  bf16 has
// no packed multiply: the group scale is applied in fp32, so the 4- and 3-bit pair tables hold their
// two values already widened to fp32 (8 bytes), which saves the two widening instructions per pair;
// the 2-bit quad table stays four 16-bit values.
template <int BITS, typename DT> struct Tab {
    static constexpr bool WIDE = false;
    static constexpr int ENTRY_BYTES = Geo<BITS>::ENTRY_BYTES;
};
template <> struct Tab<4, BF16> { static constexpr bool WIDE = true; static constexpr int ENTRY_BYTES = 8; };
template <> struct Tab<3, BF16> { static constexpr bool WIDE = true; static constexpr int ENTRY_BYTES = 8; };

// Packed words of one tile as held by one lane.
template <int BITS> struct WFrag { u32x4 w; };
template <> struct WFrag<3> { u32x4 w; u32x2 hi; };

// ---------------------------------------------------------------------------------------
// Global loads go through buffer instructions: an offset at or beyond the buffer size returns zeros
// and touches no memory.  That gives (a) the zero padding of the activation rows m >= M for free and
// (b) branch-free software pipelining: a prefetch past the end of a wave's K range is issued with an
// out-of-range offset instead of being skipped, so the instruction stream (and with it the
// compiler's wait counts) is the same on every path.
// ---------------------------------------------------------------------------------------
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr uint32_t kOutOfRange = 0x80000000u;      // every buffer is smaller than 2 GiB (checked on the host)

__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

constexpr int kAuxNone = 0;
constexpr int kAuxStream = 2;   // non-temporal: data that is read exactly once

template <int BITS>
__device__ __forceinline__ void load_wfrag(WFrag<BITS>& f, rsrc_t packed, uint32_t tile_off, int lane) {
    f.w = __builtin_amdgcn_raw_buffer_load_b128(packed, tile_off + 16u * lane, 0, kAuxStream);
    if constexpr (BITS == 3)
        f.hi = __builtin_amdgcn_raw_buffer_load_b64(packed, tile_off + 1024u + 8u * lane, 0, kAuxStream);
}

// ---------------------------------------------------------------------------------------
// Vectorised table in LDS (Section 3.2).  Entry e of copy c lives at byte
// (e << (log2c + log2 ENTRY_BYTES)) + c * ENTRY_BYTES, and lane l reads copy l mod copies, so the
// bank a lane touches depends on the lane only, never on the index: no bank conflicts.
//   4-bit: e = 8-bit pair  (q0 | q1 << 4)            -> {T[q0], T[q1]}
//   3-bit: e = 6-bit pair  (lo2(q0) | lo2(q1) << 2 | bit2(q0) << 4 | bit2(q1) << 5)
//   2-bit: e = 8-bit quad  (q0 | q1 << 2 | q2 << 4 | q3 << 6) -> {T[q0], T[q1], T[q2], T[q3]}
// With an entry stride of exactly 256 bytes (64 copies of 4 bytes, 32 copies of 8 bytes) the byte
// address is "index byte in bits 8..15, lane offset in bits 0..7", which one v_perm_b32 assembles
// straight from a packed word: one VALU instruction per lookup instead of extract + shift-add.
//
// Built without staging: entry e is a row of `stride` bytes (the same value repeated), and the
// ENTRIES rows are dealt to the threads, a power of two of threads per row (the largest that
// nthreads / ENTRIES allows; nthreads >= ENTRIES, threads left over do nothing).  Every thread fetches the one or two table
// values of its row straight from global memory (lut_fetch), and later writes its part of the row
// as 128-bit stores (lut_build).  The 16-byte chunk a lane starts with is skewed by its row number,
// so that the lanes of one store instruction, whose rows are 256 bytes apart, hit different banks.
// The two halves are separate so that the caller can issue the reads of T first, then its weight
// prefetch, and only then wait for T: lut_fetch returns the loaded words untouched.  lut_build is called by all `nthreads` threads; the caller synchronises after it.
// ---------------------------------------------------------------------------------------
struct LutSeed { uint32_t w[4]; };      // the aligned 32-bit words that hold this thread's table values

// log2 of the threads that share one row (the fused kernel gets it from the host)
template <int BITS>
__host__ __device__ constexpr int lut_log2_threads_per_row(int nthreads) {
    const int t = nthreads / Geo<BITS>::ENTRIES;
    return t >= 16 ? 4 : t >= 8 ? 3 : t >= 4 ? 2 : t >= 2 ? 1 : 0;
}

// The table indices (up to four) that entry e of the vectorised table is made of.
// pairs (4 and 2 bits): the caller's table IS the vectorised one -- a codebook of 256 pairs (4 bits: entry e = values 2e
// and 2e + 1 of the flat array) or 256 quads (2 bits: values 4e .. 4e + 3) -- instead of sixteen or four scalars that
// every nibble or bit pair of the byte is looked up in.
constexpr int kLutPairsFlag = 256;      // set in the `ltpe` argument of lut_fetch / lut_build: the table is a codebook of pairs or quads
template <int BITS>
__device__ __forceinline__ void entry_indices(int e, int q[4], bool pairs = false) {
    if constexpr (BITS == 4) {
        q[0] = pairs ? 2 * e : e & 15; q[1] = pairs ? 2 * e + 1 : (e >> 4) & 15; q[2] = 0; q[3] = 0;
    } else if constexpr (BITS == 3) {
        q[0] = (e & 3) | (((e >> 4) & 1) << 2);
        q[1] = ((e >> 2) & 3) | (((e >> 5) & 1) << 2);
        q[2] = 0; q[3] = 0;
    } else {
        q[0] = pairs ? 4 * e : e & 3; q[1] = pairs ? 4 * e + 1 : (e >> 2) & 3;
        q[2] = pairs ? 4 * e + 2 : (e >> 4) & 3; q[3] = pairs ? 4 * e + 3 : (e >> 6) & 3;
    }
}

// lut_fetch returns what it loaded untouched -- whole aligned 32-bit words, so that not even a zero
// extension follows the loads: any instruction on the loaded values would make the compiler wait for
// them right there, in front of the weight prefetch.  T needs 2-byte alignment only: the word that
// holds T[q] is word (q + mis) / 2 of the aligned address at or below T, mis = 1 if T starts in the
// upper half of a word; lut_build picks the half.
template <int BITS>
__device__ __forceinline__ LutSeed lut_fetch(const uint16_t* __restrict__ T, int tid, int ltpe) {
    const bool pairs = (ltpe & kLutPairsFlag) != 0;
    ltpe &= kLutPairsFlag - 1;
    const int e = (tid >> ltpe) & (Geo<BITS>::ENTRIES - 1);
    const uintptr_t addr = reinterpret_cast<uintptr_t>(T);
    typedef __attribute__((address_space(1))) const uint32_t global_cu32;
    global_cu32* words = reinterpret_cast<global_cu32*>(addr & ~(uintptr_t)3);
    const int mis = (int)(addr >> 1) & 1;
    int q[4];
    entry_indices<BITS>(e, q, pairs);
    LutSeed s;
#pragma unroll
    for (int i = 0; i < 4; ++i) s.w[i] = (BITS == 2 || i < 2) ? words[(q[i] + mis) >> 1] : 0u;
    return s;
}

// mis: 1 if the table's first value sits in the upper half of word 0 (a pointer that is not 4-byte aligned)
template <int BITS, typename DT>
__device__ __forceinline__ void lut_build(char* lds, const LutSeed& seed, int mis, int log2c, int tid, int ltpe) {
    using Gm = Geo<BITS>;
    constexpr int ESH = Tab<BITS, DT>::ENTRY_BYTES == 8 ? 3 : 2;
    const bool pairs = (ltpe & kLutPairsFlag) != 0;
    ltpe &= kLutPairsFlag - 1;
    const int stride = 1 << (log2c + ESH);                        // bytes of one row
    const int chunks = stride >> 4;                               // 16-byte chunks of one row (power of two)
    const int tpe = 1 << ltpe;                                    // threads per row
    const int e = tid >> ltpe, part = tid & (tpe - 1);
    const int per = chunks / tpe > 0 ? chunks / tpe : 1;          // chunks written by this thread
    if (e >= Gm::ENTRIES || part * per >= chunks) return;
    int q[4];
    entry_indices<BITS>(e, q, pairs);
    uint32_t val[4];                                              // the 16-bit table values of this row
#pragma unroll
    for (int i = 0; i < 4; ++i) val[i] = ((q[i] + mis) & 1) ? (seed.w[i] >> 16) : (seed.w[i] & 0xffffu);
    u32x4 v;
    if constexpr (Tab<BITS, DT>::WIDE) {          // {T[q0], T[q1]} as fp32
        v.x = val[0] << 16; v.y = val[1] << 16; v.z = v.x; v.w = v.y;
    } else {
        v.x = val[0] | (val[1] << 16);
        if constexpr (Gm::ENTRY_BYTES == 8) { v.y = val[2] | (val[3] << 16); v.z = v.x; v.w = v.y; }
        else { v.y = v.x; v.z = v.x; v.w = v.x; }
    }
    char* row = lds + (size_t)e * stride;
#pragma unroll 1
    for (int i = 0; i < per; ++i) {
        const int c = (part * per + i + e) & (chunks - 1);
        *reinterpret_cast<u32x4*>(row + 16 * c) = v;
    }
}

template <int BITS, typename DT>
__device__ __forceinline__ void build_lut(char* lds, const uint16_t* __restrict__ T, int log2c, int tid, int nthreads) {
    const int ltpe = lut_log2_threads_per_row<BITS>(nthreads);
    const LutSeed s = lut_fetch<BITS>(T, tid, ltpe);
    lut_build<BITS, DT>(lds, s, (int)(reinterpret_cast<uintptr_t>(T) >> 1) & 1, log2c, tid, ltpe);
}

// ---------------------------------------------------------------------------------------
// One table per output row (finer-grained tables: every output channel has its own 2^b values).
// A lane only ever looks up indices of one row of a row block (row lane % 16), so its private copy of
// the table can simply hold that row's table and the lookup code does not change.  The copies of a
// row block are rebuilt whenever a workgroup moves to another row block: every lane fetches its
// row's 2^b values (rowlut_fetch, issued before the weight prefetch), then the waves deal the
// entries between them by their upper index (wave w takes upper indices w, w + nw, w + 2 nw, w + 3 nw;
// nw >= 4) and each lane writes its own copy of those entries (rowlut_build).  Entry contents and
// the 256-byte entry stride are those of lut_build.
// ---------------------------------------------------------------------------------------
struct RowTab { u32x4 a, b; };           // the row's 2^b 16-bit values, two per word

template <int BITS>
__device__ __forceinline__ RowTab rowlut_fetch(const uint16_t* __restrict__ T, int64_t row) {
    RowTab t;
    t.a = u32x4{0, 0, 0, 0}; t.b = t.a;
    const uint16_t* src = T + row * (1 << BITS);
    if constexpr (BITS == 4) {
        t.a = *reinterpret_cast<const u32x4*>(src);
        t.b = *reinterpret_cast<const u32x4*>(src + 8);
    } else if constexpr (BITS == 3) {
        t.a = *reinterpret_cast<const u32x4*>(src);
    } else {
        const u32x2 v = *reinterpret_cast<const u32x2*>(src);
        t.a.x = v.x; t.a.y = v.y;
    }
    return t;
}

template <int BITS, typename DT>
__device__ __forceinline__ void rowlut_build(char* lds, const RowTab& t, int wave, int nw, int lane) {
    auto val = [&](int q) -> uint32_t {                   // value q of the row's table (q is a constant)
        const uint32_t w = q / 2 < 4 ? t.a[q / 2] : t.b[q / 2 - 4];
        return (q & 1) ? (w >> 16) : (w & 0xffffu);
    };
    const int w1 = wave + nw, w2 = wave + 2 * nw, w3 = wave + 3 * nw;
    constexpr bool WIDE = Tab<BITS, DT>::WIDE;
    constexpr int UPPER = BITS == 3 ? 8 : 16;             // upper indices (4-bit: q1; 3-bit: q1; 2-bit: (q3, q2))
    constexpr int LOWER = BITS == 3 ? 8 : 16;
#pragma unroll
    for (int hi = 0; hi < UPPER; ++hi) {
        if (!(hi == wave || hi == w1 || hi == w2 || hi == w3)) continue;
#pragma unroll
        for (int lo = 0; lo < LOWER; ++lo) {
            if constexpr (BITS == 4) {
                const int e = lo | (hi << 4);
                if constexpr (WIDE) {
                    if (lane < 32) *reinterpret_cast<u32x2*>(lds + e * 256 + lane * 8) = u32x2{val(lo) << 16, val(hi) << 16};
                } else {
                    *reinterpret_cast<uint32_t*>(lds + e * 256 + lane * 4) = val(lo) | (val(hi) << 16);
                }
            } else if constexpr (BITS == 3) {
                const int e = (lo & 3) | ((hi & 3) << 2) | ((lo >> 2) << 4) | ((hi >> 2) << 5);
                if constexpr (WIDE) {
                    if (lane < 32) *reinterpret_cast<u32x2*>(lds + e * 256 + lane * 8) = u32x2{val(lo) << 16, val(hi) << 16};
                } else {
                    *reinterpret_cast<uint32_t*>(lds + e * 256 + lane * 4) = val(lo) | (val(hi) << 16);
                }
            } else {
                const int e = lo | (hi << 4);
                if (lane < 32)
                    *reinterpret_cast<u32x2*>(lds + e * 256 + lane * 8) =
                        u32x2{val(lo & 3) | (val((lo >> 2) & 3) << 16), val(hi & 3) | (val((hi >> 2) & 3) << 16)};
            }
        }
    }
}

template <int BITS, typename DT>
__host__ __device__ constexpr int lut_lds_bytes(int log2c) {
    return (Geo<BITS>::ENTRIES * Tab<BITS, DT>::ENTRY_BYTES) << log2c;
}
// log2 of the number of copies that makes the entry stride 256 bytes
template <int BITS, typename DT>
__host__ __device__ constexpr int perm_log2_copies() {
    return Tab<BITS, DT>::ENTRY_BYTES == 8 ? 5 : 6;
}

// ---------------------------------------------------------------------------------------
// Per-row tables, sixteen copies: the table of row c of a row block is copy c (log2 copies = 4), so
// lane l reads copy l % 16 = its row, with the generic (shift + add) entry address.
// ---------------------------------------------------------------------------------------
template <int BITS, typename DT>
__host__ __device__ constexpr int rowlut16_bytes() { return lut_lds_bytes<BITS, DT>(4); }
// bytes of one row block's raw tables (16 rows x 2^b 16-bit values), staged in LDS for the build
template <int BITS>
__host__ __device__ constexpr int rowlut16_stage_bytes() { return 16 * (1 << BITS) * 2; }

// Builds the tables of `nrb` row blocks at `tables` (rowlut16_bytes apart) from their raw rows at `stage`
// (both LDS).  Thread (row block a, row c, lower index lo) reads the row's 2^b values once and writes the
// entries (lo, hi) for every upper index hi: the lanes of one store cover rows c = 0..15 (one entry's
// sixteen copies, contiguous) of four consecutive entries, so stores do not conflict.
template <int BITS, typename DT>
__device__ __forceinline__ void rowlut16_build(char* tables, const char* stage, int nrb, int tid, int nthreads) {
    constexpr int E = 1 << BITS;
    constexpr int LOWN = BITS == 3 ? 8 : 16, LOWL = BITS == 3 ? 3 : 4;
    constexpr bool WIDE = Tab<BITS, DT>::WIDE;
    constexpr int EB = Tab<BITS, DT>::ENTRY_BYTES;
    constexpr int SH = 4 + (EB == 8 ? 3 : 2);
    const int combos = nrb * 16 * LOWN;
    for (int idx = tid; idx < combos; idx += nthreads) {
        const int c = idx & 15, lo = (idx >> 4) & (LOWN - 1), a = idx >> (4 + LOWL);
        const char* row = stage + (size_t)(a * 16 + c) * (E * 2);
        uint32_t t[8] = {0, 0, 0, 0, 0, 0, 0, 0};               // the row's values, two per word
        if constexpr (BITS == 4) {
            const u32x4 v0 = *reinterpret_cast<const u32x4*>(row), v1 = *reinterpret_cast<const u32x4*>(row + 16);
            t[0] = v0.x; t[1] = v0.y; t[2] = v0.z; t[3] = v0.w; t[4] = v1.x; t[5] = v1.y; t[6] = v1.z; t[7] = v1.w;
        } else if constexpr (BITS == 3) {
            const u32x4 v0 = *reinterpret_cast<const u32x4*>(row);
            t[0] = v0.x; t[1] = v0.y; t[2] = v0.z; t[3] = v0.w;
        } else {
            const u32x2 v0 = *reinterpret_cast<const u32x2*>(row);
            t[0] = v0.x; t[1] = v0.y;
        }
        auto val = [&](int q) -> uint32_t { return (q & 1) ? (t[q >> 1] >> 16) : (t[q >> 1] & 0xffffu); };   // q is a constant
        const uint16_t* rowv = reinterpret_cast<const uint16_t*>(row);
        uint32_t first;                                         // the part of the entry that lo decides
        int e_lo;
        if constexpr (BITS == 2) {
            first = (uint32_t)rowv[lo & 3] | ((uint32_t)rowv[lo >> 2] << 16);
            e_lo = lo;
        } else {
            first = rowv[lo];
            e_lo = BITS == 3 ? ((lo & 3) | ((lo >> 2) << 4)) : lo;
        }
        char* dst = tables + (size_t)a * rowlut16_bytes<BITS, DT>() + ((size_t)e_lo << SH) + c * EB;
#pragma unroll
        for (int hi = 0; hi < LOWN; ++hi) {
            const int e_hi = BITS == 3 ? (((hi & 3) << 2) | ((hi >> 2) << 5)) : (hi << 4);
            if constexpr (BITS == 2) {
                *reinterpret_cast<u32x2*>(dst + (e_hi << SH)) = u32x2{first, val(hi & 3) | (val(hi >> 2) << 16)};
            } else if constexpr (WIDE) {
                *reinterpret_cast<u32x2*>(dst + (e_hi << SH)) = u32x2{first << 16, val(hi) << 16};
            } else {
                *reinterpret_cast<uint32_t*>(dst + (e_hi << SH)) = first | (val(hi) << 16);
            }
        }
    }
}

// bytes of the fused kernel's table: every entry is one 256-byte row, whatever it holds
template <int BITS>
__host__ __device__ constexpr int lut_row_table_bytes() { return Geo<BITS>::ENTRIES * 256; }

typedef __attribute__((address_space(3))) const uint32_t lds_cu32;
typedef __attribute__((address_space(3))) const u32x2 lds_cu64;

// Per-lane constants of the lookup: the shift that turns an entry number into a byte offset, and
// the LDS byte address of entry 0 of this lane's private copy (table base included; for the
// v_perm form the table must start at LDS address 0, which it does as the first dynamic array).
struct LutAddr {
    int sh;
    uint32_t lane_base;
};
template <int BITS, typename DT>
__device__ __forceinline__ LutAddr make_lut_addr(const char* lut_lds, int log2c, int lane) {
    LutAddr a;
    a.sh = log2c + (Tab<BITS, DT>::ENTRY_BYTES == 8 ? 3 : 2);
    const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)lut_lds;
    a.lane_base = base + (uint32_t)(lane & ((1 << log2c) - 1)) * Tab<BITS, DT>::ENTRY_BYTES;
    return a;
}

// Address of the entry selected by byte `p` of `word`.  PERM: bytes {lane_base.0, word.p, lane_base.2,
// lane_base.3}; v_perm_b32 numbers the bytes of its second operand 0..3 and of its first 4..7.
template <bool PERM, int P>
__device__ __forceinline__ uint32_t entry_addr(uint32_t word, LutAddr la) {
    if constexpr (PERM) {
        return __builtin_amdgcn_perm(word, la.lane_base, 0x03020000u | ((4u + P) << 8));
    } else {
        const uint32_t idx = (P == 3) ? (word >> 24) : ((word >> (8 * P)) & 0xffu);
        return (idx << la.sh) + la.lane_base;
    }
}
__device__ __forceinline__ uint32_t lds_u32(uint32_t addr) {
    return *reinterpret_cast<lds_cu32*>((uintptr_t)addr);
}
__device__ __forceinline__ u32x2 lds_u64(uint32_t addr) {
    return *reinterpret_cast<lds_cu64*>((uintptr_t)addr);
}

// ---------------------------------------------------------------------------------------
// Group scale.  fp16: one packed half multiply per pair.  bf16: widen both halves to fp32 (exact),
// multiply (exact: 8 x 8 significand bits), round once to bf16 (round-to-nearest-even).
// Both give round16(T[q] * s) with a single rounding.
// ---------------------------------------------------------------------------------------
template <typename DT> struct ScaleReg;
template <> struct ScaleReg<F16> { uint32_t s2; };    // scale in both halves
template <> struct ScaleReg<BF16> { float s; };

// Scale register from 16-bit half `hi` (0: low, 1: high) of a 32-bit word: one instruction each.
template <typename DT> __device__ __forceinline__ ScaleReg<DT> make_scale(uint32_t word, int hi);
template <> __device__ __forceinline__ ScaleReg<F16> make_scale<F16>(uint32_t w, int hi) {
    ScaleReg<F16> r; r.s2 = __builtin_amdgcn_perm(w, w, hi ? 0x03020302u : 0x01000100u); return r;
}
template <> __device__ __forceinline__ ScaleReg<BF16> make_scale<BF16>(uint32_t w, int hi) {
    ScaleReg<BF16> r; r.s = __builtin_bit_cast(float, hi ? (w & 0xffff0000u) : (w << 16)); return r;
}

__device__ __forceinline__ uint32_t scale_pair(uint32_t pair, ScaleReg<F16> s) {
    f16x2 v = __builtin_bit_cast(f16x2, pair) * __builtin_bit_cast(f16x2, s.s2);
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint32_t scale_pair(uint32_t pair, ScaleReg<BF16> s) {
    f32x2 v;
    v.x = __builtin_bit_cast(float, pair << 16) * s.s;
    v.y = __builtin_bit_cast(float, pair & 0xffff0000u) * s.s;
    bf16x2 r = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, r);
}

// ---------------------------------------------------------------------------------------
// One 32-wide K step of one 16-row block.  lookup_step issues the table reads for this lane's 8
// weights (unscaled, four 32-bit registers in A-operand order); scale4 applies the group scale.
// They are separate so that the caller can issue the LDS reads of the next step before it consumes
// the current one.
// ---------------------------------------------------------------------------------------
// Unscaled table values of one step: four registers (16-bit pairs in A-operand order), or, for the
// widened bf16 tables, eight fp32 values.
template <int BITS, typename DT> struct Raw { u32x4 v; };
template <> struct Raw<4, BF16> { u32x4 even, odd; };    // values 2p (even) and 2p + 1 (odd), p = 0..3
template <> struct Raw<3, BF16> { u32x4 even, odd; };

// The four table addresses of a step come from the four bytes of one 32-bit word of indices.
template <int BITS>
__device__ __forceinline__ uint32_t index_word(const WFrag<BITS>& f, int step) {
    if constexpr (BITS == 4) {
        return f.w[step];
    } else if constexpr (BITS == 3) {
        // combine the two bit-slices: bits 0..3 of each byte from the low slice, bits 4..5 from the
        // high slice, bits 6..7 cleared: four 6-bit pair-table indices, one per byte.
        const uint32_t lo = (step & 1) ? (f.w[step >> 1] >> 4) : f.w[step >> 1];
        const int u = step & 3;
        const uint32_t h = f.hi[step >> 2];
        const uint32_t hs = (u == 0) ? (h << 4) : (u == 1) ? (h << 2) : (u == 2) ? h : (h >> 2);
        return (hs & 0x30303030u) | (lo & 0x0f0f0f0fu);
    } else {
        return f.w[step >> 1];             // two steps per word: bytes 0,1 and 2,3
    }
}

template <int BITS, typename DT, bool PERM>
__device__ __forceinline__ Raw<BITS, DT> lookup_step(const WFrag<BITS>& f, int step, LutAddr la) {
    Raw<BITS, DT> a;
    const uint32_t w = index_word<BITS>(f, step);
    if constexpr (Tab<BITS, DT>::WIDE) {
        const u32x2 p0 = lds_u64(entry_addr<PERM, 0>(w, la));
        const u32x2 p1 = lds_u64(entry_addr<PERM, 1>(w, la));
        const u32x2 p2 = lds_u64(entry_addr<PERM, 2>(w, la));
        const u32x2 p3 = lds_u64(entry_addr<PERM, 3>(w, la));
        a.even = u32x4{p0.x, p1.x, p2.x, p3.x};
        a.odd = u32x4{p0.y, p1.y, p2.y, p3.y};
    } else if constexpr (BITS == 2) {
        const u32x2 q0 = (step & 1) ? lds_u64(entry_addr<PERM, 2>(w, la)) : lds_u64(entry_addr<PERM, 0>(w, la));
        const u32x2 q1 = (step & 1) ? lds_u64(entry_addr<PERM, 3>(w, la)) : lds_u64(entry_addr<PERM, 1>(w, la));
        a.v.x = q0.x; a.v.y = q0.y; a.v.z = q1.x; a.v.w = q1.y;
    } else {
        a.v.x = lds_u32(entry_addr<PERM, 0>(w, la));
        a.v.y = lds_u32(entry_addr<PERM, 1>(w, la));
        a.v.z = lds_u32(entry_addr<PERM, 2>(w, la));
        a.v.w = lds_u32(entry_addr<PERM, 3>(w, la));
    }
    return a;
}

// Group scale applied to the eight values of a step; result in A-operand order.  Each product is
// rounded once to the 16-bit type (fp16: packed half multiply; bf16: exact fp32 product, one conversion).
template <int BITS, typename DT>
__device__ __forceinline__ u32x4 scale4(const Raw<BITS, DT>& raw, ScaleReg<DT> sc) {
    u32x4 a;
    if constexpr (Tab<BITS, DT>::WIDE) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t e = raw.even[j], o = raw.odd[j];
            f32x2 v;
            v.x = __builtin_bit_cast(float, e) * sc.s;
            v.y = __builtin_bit_cast(float, o) * sc.s;
            a[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
        }
    } else {
        a.x = scale_pair(raw.v.x, sc);
        a.y = scale_pair(raw.v.y, sc);
        a.z = scale_pair(raw.v.z, sc);
        a.w = scale_pair(raw.v.w, sc);
    }
    return a;
}

// Lane i of every 16-lane row receives the value of lane (i + n) mod 16 of the same row
// (a DPP row rotate to the right by 16 - n lanes), for each of the four registers; n in {0, 4, 8, 12}.
// A rotation reads a valid lane for every lane, so the destination needs no previous value.
template <int CTRL>
__device__ __forceinline__ u32x4 dpp4(u32x4 v) {
    u32x4 r;
    r.x = (uint32_t)__builtin_amdgcn_mov_dpp((int)v.x, CTRL, 0xf, 0xf, true);
    r.y = (uint32_t)__builtin_amdgcn_mov_dpp((int)v.y, CTRL, 0xf, 0xf, true);
    r.z = (uint32_t)__builtin_amdgcn_mov_dpp((int)v.z, CTRL, 0xf, 0xf, true);
    r.w = (uint32_t)__builtin_amdgcn_mov_dpp((int)v.w, CTRL, 0xf, 0xf, true);
    return r;
}
__device__ __forceinline__ u32x4 rotate_rows(u32x4 v, int n) {
    switch (n) {                       // row_ror:k is control 0x120 + k
        case 4: return dpp4<0x120 + 12>(v);
        case 8: return dpp4<0x120 + 8>(v);
        case 12: return dpp4<0x120 + 4>(v);
        default: return v;
    }
}

// v_mfma_f32_16x16x32: D(16x16, fp32) += A(16x32) * B(32x16).  Lane l = 16*o + i supplies A[i][8o..8o+7]
// and B[8o..8o+7][i]; it receives D[4o..4o+3][i].
template <typename DT>
__device__ __forceinline__ f32x4 mfma16x16x32(u32x4 a, u32x4 b, f32x4 c);
template <>
__device__ __forceinline__ f32x4 mfma16x16x32<F16>(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <>
__device__ __forceinline__ f32x4 mfma16x16x32<BF16>(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// fp32 -> 16-bit, round-to-nearest-even, four values packed into 8 bytes.
template <typename DT> __device__ __forceinline__ u32x2 pack4(f32x4 v);
template <> __device__ __forceinline__ u32x2 pack4<F16>(f32x4 v) {
    f16x4 h = __builtin_convertvector(v, f16x4);
    return __builtin_bit_cast(u32x2, h);
}
template <> __device__ __forceinline__ u32x2 pack4<BF16>(f32x4 v) {
    bf16x4 h = __builtin_convertvector(v, bf16x4);
    return __builtin_bit_cast(u32x2, h);
}

// Scales of one tile for one row: NS = TK / GROUP consecutive 16-bit values, loaded as one access.
template <int NS> struct ScaleWords { uint32_t w[(NS + 1) / 2]; };

template <int NS>
__device__ __forceinline__ void load_scales(ScaleWords<NS>& s, rsrc_t scales, uint32_t byte_off) {
    if constexpr (NS == 1) s.w[0] = __builtin_amdgcn_raw_buffer_load_b16(scales, byte_off, 0, kAuxNone);
    else if constexpr (NS == 2) s.w[0] = __builtin_amdgcn_raw_buffer_load_b32(scales, byte_off, 0, kAuxNone);
    else if constexpr (NS == 4) {
        u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(scales, byte_off, 0, kAuxNone);
        s.w[0] = v.x; s.w[1] = v.y;
    } else {
        u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(scales, byte_off, 0, kAuxNone);
        s.w[0] = v.x; s.w[1] = v.y; s.w[2] = v.z; s.w[3] = v.w;
    }
}
template <int NS>
__device__ __forceinline__ void lds_load_scales(ScaleWords<NS>& s, const char* p) {
    if constexpr (NS == 1) s.w[0] = *reinterpret_cast<const uint16_t*>(p);
    else if constexpr (NS == 2) s.w[0] = *reinterpret_cast<const uint32_t*>(p);
    else if constexpr (NS == 4) {
        u32x2 v = *reinterpret_cast<const u32x2*>(p);
        s.w[0] = v.x; s.w[1] = v.y;
    } else {
        u32x4 v = *reinterpret_cast<const u32x4*>(p);
        s.w[0] = v.x; s.w[1] = v.y; s.w[2] = v.z; s.w[3] = v.w;
    }
}
template <typename DT, int NS>
__device__ __forceinline__ ScaleReg<DT> scale_of(const ScaleWords<NS>& s, int g) {
    return make_scale<DT>(s.w[g >> 1], g & 1);
}

}  // namespace lutq
