// Offline restructuring of the index matrix (Section 3.1 of the paper: reorder the
// static quantised weights once so that, after dequantisation, registers already hold
// the matrix-instruction operand layout; split 3-bit indices into a 2-bit and a 1-bit
// slice so that all loads are a power-of-two number of bits).
//
// The byte layout is specified in include/lutq.h ("Packed layout"); its geometry is lutq_layout.hpp.
#include "lutq.h"
#include "lutq_layout.hpp"

#include <cstring>

namespace {

using lutq::layout::super_block;
using lutq::layout::tile_bytes;
using lutq::layout::tile_index;
using lutq::layout::tile_k;

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

extern "C" lutq_status lutq_pack_layout(int64_t N, int64_t K, int bits, int group_size, lutq_layout* out) {
    if (!out) return LUTQ_ERR_NULL;
    const lutq_status st = check_pack_args(N, K, bits, group_size);
    if (st != LUTQ_OK) return st;
    out->tile_k = tile_k(bits);
    out->tile_bytes = tile_bytes(bits);
    out->row_blocks_per_super_block = super_block(N / 16);
    out->row_blocks = N / 16;
    out->k_tiles = K / tile_k(bits);
    return LUTQ_OK;
}

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
