// The geometry of the packed weight layout, defined once for the packer, the GPU quantiser and the
// launch code (the byte layout itself is specified in include/lutq.h).
#pragma once

#include <stdint.h>

namespace lutq {
namespace layout {

// K columns and bytes of one tile (what one wavefront loads with one 128-bit load per lane, plus one
// 64-bit load for the 3-bit high slice)
inline int tile_k(int bits) { return bits == 4 ? 128 : 256; }
inline int tile_bytes(int bits) { return bits == 3 ? 1536 : 1024; }

// Row blocks per super-block, from the number of 16-row blocks nb = N / 16: 4 where nb is a multiple
// of 4, else 2 where it is even, else 1 -- except 2 for multiples of 4 in 257..512.  The exception is a
// tuning choice for 256 compute units that is frozen into the format: with between one and two row
// blocks per compute unit a workgroup streams two row blocks, and a super-block of 2 makes those one
// contiguous run of memory (N = K = 8192, M = 1: 8.90 us against 9.96 us with super-blocks of 4).  It
// is part of the layout whatever the device; lutq_pack_layout reports the value for a given N.
inline int super_block(int64_t nb) { return (nb % 4 == 0 && (nb <= 256 || nb > 512)) ? 4 : nb % 2 == 0 ? 2 : 1; }

// index of tile (row block rb, K tile kt) in storage order: super-block, K tile, row block inside it
inline int64_t tile_index(int64_t rb, int64_t kt, int64_t KT, int SB) { return ((rb / SB) * KT + kt) * SB + rb % SB; }

}  // namespace layout
}  // namespace lutq
