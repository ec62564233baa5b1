// Offline restructuring of the index matrix (Section 3.1 of the paper: reorder the
// static quantised weights once so that, after dequantisation, registers already hold
// the matrix-instruction operand layout; split 3-bit indices into a 2-bit and a 1-bit
// slice so that all loads are a power-of-two number of bits).
//
// Packed layout (this library's own; the paper's is tied to NVIDIA Ampere fragments).
//
// Q is [N, K] row-major.  N is cut into row blocks of 16 rows, K into tiles of TK columns
// (TK = 128 for 4-bit, 256 for 2- and 3-bit).  Row blocks are grouped into super-blocks of SB
// consecutive row blocks (SB = 4 if N/16 is a multiple of 4 and not in 257..512, else 2 if N/16 is even,
// else 1; see super_block below).  Storage order is
// super-block, then K tile, then row block inside the super-block: tile (rb, kt) starts at byte
//        (((rb / SB) * K/TK + kt) * SB + rb % SB) * TILE_BYTES,
// so the SB tiles that cover 16*SB rows x TK columns are adjacent: a wavefront that owns a whole
// super-block streams one contiguous run of memory along K instead of SB separate runs.  A tile is
// what one 64-lane wavefront loads with one 128-bit load per lane (plus one 64-bit load for the
// 3-bit high slice).
//
// The gfx950 instruction v_mfma_f32_16x16x32_{f16,bf16} takes, from lane l = 16*o + i
// (i = 0..15, o = 0..3), the eight A-matrix elements of row i and columns 8*o .. 8*o+7
// of a 16 x 32 block.  A K tile holds TK/32 such blocks ("steps" t).  Lane l therefore
// owns, for step t, the indices
//        Q[16*rb + i][TK*kt + 32*t + 8*o + j],   j = 0..7,
// and its bytes sit at offset 16*l of the tile:
//
//  4-bit  TILE_BYTES = 1024.  Four little-endian 32-bit words d = 0..3; word d is step d;
//         nibble j (bits 4j..4j+3) is index j.  Byte p of a word is thus the pair
//         (j = 2p, 2p+1): directly the address of a pair-table entry.
//  2-bit  TILE_BYTES = 1024.  Words d = 0..3; 2-bit field e (bits 2e..2e+1), e = 0..15, of
//         word d is index j = e % 8 of step t = 2d + e / 8.  Byte p holds four consecutive
//         indices: the address of a quad-table entry.
//  3-bit  TILE_BYTES = 1536 = 1024 (low slice: index bits 0..1) + 512 (high slice: bit 2).
//         Low slice, lane l at 16*l, words d = 0..3, byte p = 0..3 of word d:
//              bits 0..1 low2(index 2p, step 2d)      bits 2..3 low2(index 2p+1, step 2d)
//              bits 4..5 low2(index 2p, step 2d+1)    bits 6..7 low2(index 2p+1, step 2d+1)
//         High slice, lane l at 1024 + 8*l, words h = 0..1, byte p of word h, u = 0..3:
//              bit 2u   = bit2(index 2p,   step 4h+u)
//              bit 2u+1 = bit2(index 2p+1, step 4h+u)
//         so that, for one step, (low word >> 0 or 4) supplies bits 0..3 of each byte and
//         (high word shifted by 4 - 2u) supplies bits 4..5: four 6-bit pair-table addresses.
#include "lutq.h"

#include <cstring>

namespace {

inline int tile_k(int bits) { return bits == 4 ? 128 : 256; }
inline int tile_bytes(int bits) { return bits == 3 ? 1536 : 1024; }
// Between one and two row blocks per compute unit of the 256-CU part (N/16 in 257..512) a workgroup
// streams two row blocks: with SB = 2 these two are one contiguous run of memory (measured on
// N = K = 8192, M = 1: 9.96 us with SB = 4, 8.90 us with SB = 2); everywhere else SB = 4 measured best.
inline int super_block(int64_t nb) { return (nb % 4 == 0 && (nb <= 256 || nb > 512)) ? 4 : nb % 2 == 0 ? 2 : 1; }
inline int64_t tile_index(int64_t rb, int64_t kt, int64_t KT, int SB) { return ((rb / SB) * KT + kt) * SB + rb % SB; }

lutq_status check_pack_args(int64_t N, int64_t K, int bits, int group_size) {
    if (bits < 2 || bits > 4) return LUTQ_ERR_BITS;
    if (group_size != 32 && group_size != 64 && group_size != 128 && group_size != 256) return LUTQ_ERR_GROUP;
    if (N <= 0 || K <= 0 || N % 16 != 0 || K % tile_k(bits) != 0) return LUTQ_ERR_SHAPE;
    if (K % group_size != 0) return LUTQ_ERR_GROUP;
    return LUTQ_OK;
}

inline void put_bits(uint8_t* tile, int byte_off, int bit, uint32_t v) {
    // little-endian 32-bit word at byte_off, bit position `bit` (field never straddles a byte)
    tile[byte_off + (bit >> 3)] |= (uint8_t)(v << (bit & 7));
}

inline uint32_t get_bits(const uint8_t* tile, int byte_off, int bit, int width) {
    return (tile[byte_off + (bit >> 3)] >> (bit & 7)) & ((1u << width) - 1u);
}

// Location of index (step t, element j) of lane l inside a tile.
struct Loc { int byte_off; int bit; };
inline Loc loc4(int l, int t, int j) { return { 16 * l + 4 * t, 4 * j }; }
inline Loc loc2(int l, int t, int j) { return { 16 * l + 4 * (t >> 1), 2 * (8 * (t & 1) + j) }; }
inline Loc loc3_low(int l, int t, int j) { return { 16 * l + 4 * (t >> 1), 8 * (j >> 1) + 4 * (t & 1) + 2 * (j & 1) }; }
inline Loc loc3_high(int l, int t, int j) { return { 1024 + 8 * l + 4 * (t >> 2), 8 * (j >> 1) + 2 * (t & 3) + (j & 1) }; }

}  // namespace

extern "C" size_t lutq_packed_bytes(int64_t N, int64_t K, int bits, int group_size) {
    if (check_pack_args(N, K, bits, group_size) != LUTQ_OK) return 0;
    return (size_t)(N / 16) * (size_t)(K / tile_k(bits)) * (size_t)tile_bytes(bits);
}

extern "C" lutq_status lutq_pack(const uint8_t* indices, int64_t N, int64_t K, int bits, int group_size,
                                 void* packed_out) {
    if (!indices || !packed_out) return LUTQ_ERR_NULL;
    lutq_status st = check_pack_args(N, K, bits, group_size);
    if (st != LUTQ_OK) return st;
    const int TK = tile_k(bits), TB = tile_bytes(bits), steps = TK / 32;
    const int64_t NB = N / 16, KT = K / TK;
    const int SB = super_block(NB);
    const uint32_t limit = 1u << bits;
    uint8_t* out = static_cast<uint8_t*>(packed_out);
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t rb = 0; rb < NB; ++rb) {
        for (int64_t kt = 0; kt < KT; ++kt) {
            uint8_t* tile = out + tile_index(rb, kt, KT, SB) * TB;
            std::memset(tile, 0, TB);
            for (int l = 0; l < 64; ++l) {
                const int i = l & 15, o = l >> 4;
                const uint8_t* row = indices + (16 * rb + i) * K + kt * TK + 8 * o;
                for (int t = 0; t < steps; ++t) {
                    for (int j = 0; j < 8; ++j) {
                        const uint32_t q = row[32 * t + j];
                        if (q >= limit) { bad = 1; continue; }
                        if (bits == 4) {
                            Loc a = loc4(l, t, j); put_bits(tile, a.byte_off, a.bit, q);
                        } else if (bits == 2) {
                            Loc a = loc2(l, t, j); put_bits(tile, a.byte_off, a.bit, q);
                        } else {
                            Loc a = loc3_low(l, t, j); put_bits(tile, a.byte_off, a.bit, q & 3u);
                            Loc b = loc3_high(l, t, j); put_bits(tile, b.byte_off, b.bit, q >> 2);
                        }
                    }
                }
            }
        }
    }
    return bad ? LUTQ_ERR_INDEX_RANGE : LUTQ_OK;
}

extern "C" lutq_status lutq_unpack(const void* packed, int64_t N, int64_t K, int bits, int group_size,
                                   uint8_t* indices_out) {
    if (!packed || !indices_out) return LUTQ_ERR_NULL;
    lutq_status st = check_pack_args(N, K, bits, group_size);
    if (st != LUTQ_OK) return st;
    const int TK = tile_k(bits), TB = tile_bytes(bits), steps = TK / 32;
    const int64_t NB = N / 16, KT = K / TK;
    const int SB = super_block(NB);
    const uint8_t* in = static_cast<const uint8_t*>(packed);
#pragma omp parallel for schedule(static)
    for (int64_t rb = 0; rb < NB; ++rb) {
        for (int64_t kt = 0; kt < KT; ++kt) {
            const uint8_t* tile = in + tile_index(rb, kt, KT, SB) * TB;
            for (int l = 0; l < 64; ++l) {
                const int i = l & 15, o = l >> 4;
                uint8_t* row = indices_out + (16 * rb + i) * K + kt * TK + 8 * o;
                for (int t = 0; t < steps; ++t) {
                    for (int j = 0; j < 8; ++j) {
                        uint32_t q;
                        if (bits == 4) {
                            Loc a = loc4(l, t, j); q = get_bits(tile, a.byte_off, a.bit, 4);
                        } else if (bits == 2) {
                            Loc a = loc2(l, t, j); q = get_bits(tile, a.byte_off, a.bit, 2);
                        } else {
                            Loc a = loc3_low(l, t, j); Loc b = loc3_high(l, t, j);
                            q = get_bits(tile, a.byte_off, a.bit, 2) | (get_bits(tile, b.byte_off, b.bit, 1) << 2);
                        }
                        row[32 * t + j] = (uint8_t)q;
                    }
                }
            }
        }
    }
    return LUTQ_OK;
}
