"""CPU oracle for the LUT-quantised matmul.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this file; the product (the HIP library and its Python binding) never
does, and shares no code with it.

What the path computes is an exact definition, not an approximation, so the
oracle is that definition written out in numpy with fp64 arithmetic:

  * dequantise   W^[n, k] = T[Q[n, k]]                      (Section 3, second equation)
  * group scale  W^[n, k] = T[Q[n, k]] * S[n, k // B]        (Section 4.1 "LUT quantization
    method": the group-level table is s_g * T; Section 4.2 last sentence)
  * matmul       Y = X * W^ (Section 3, objective), with W^ held as [N, K] (one
    row per output channel) so that Y[m, n] = sum_k X[m, k] * W^[n, k].

Readings of the paper taken here:
  * Orientation: the paper writes Q, W as k x n and Y = X W^; this code stores the
    transposes ([N, K], the layout of a linear layer's weight), same function.
  * The printed scale subscript "(i x j) mod B" cannot enumerate kn/B groups; a
    group is B consecutive elements along K inside one output row, so the scale
    of W^[n, k] is S[n, k // B] with S of shape [N, K / B].
  * T[q] * s is rounded once, round-to-nearest-even, to the 16-bit storage type
    (the product of two fp16 or two bf16 numbers is exact in fp64).
  * Y is accumulated in fp64 and is NOT rounded to 16 bits.

Parity pins (see tests/test_oracle_pins.py): exact rational brute force on tiny
inputs, closed forms (all-ones table, one-hot X, uniform-integer table = int-b
group quantisation), forward-CDF check and structural invariants of the
NormalFloat table, bijection of the packed layout.  The packed byte layout
itself is this project's own definition (the paper states its goal, not its
bytes): parity unpinned by the paper for `pack`; it is pinned as a bijection
whose inverse feeds the pinned dequantise + matmul.

16-bit tensors are uint16 bit patterns with a dtype tag "f16" / "bf16".
"""
from __future__ import annotations

import numpy as np
from scipy.special import ndtri

# ----------------------------------------------------------------------------
# 16-bit formats
# ----------------------------------------------------------------------------

def to_f64(bits, dtype: str) -> np.ndarray:
    """Widen fp16 / bf16 bit patterns to float64 (exact)."""
    b = np.ascontiguousarray(np.asarray(bits, dtype=np.uint16))
    if dtype == "f16":
        return b.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def from_f64(x, dtype: str) -> np.ndarray:
    """Round float64 values once, to nearest even, to fp16 / bf16 bit patterns.

    fp16: numpy converts float64 -> float16 with a single correct rounding.
    bf16: the value is scaled by a power of two so that one unit equals the bf16
    spacing at its magnitude (8 significant bits; spacing 2^-133 below 2^-126),
    rounded to the nearest even integer, and scaled back; the result is exactly
    a bf16 number, so taking the upper half of its float32 pattern is exact.
    """
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f16":
        return np.ascontiguousarray(x.astype(np.float16)).view(np.uint16)
    if dtype == "bf16":
        _, e = np.frexp(x)                                  # |x| = m * 2^e, 0.5 <= m < 1
        q = np.maximum(e - 8, -133).astype(np.float64)
        r = np.rint(x / np.exp2(q)) * np.exp2(q)
        r32 = r.astype(np.float32)                          # exact (overflow -> inf, as bf16 would)
        return (np.ascontiguousarray(r32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
# NormalFloat table (Section 4.2, first paragraph)
# ----------------------------------------------------------------------------
NF_DELTA = 0.5 * (1.0 / 30.0 + 1.0 / 32.0)


def nf_probabilities(bits: int) -> np.ndarray:
    """The 2^b probabilities p_0 = delta, ..., p_{2^(b-1)-1} = 1/2, ..., p_{2^b-1} = 1 - delta.

    2^(b-1) evenly spaced points on [delta, 1/2] and 2^(b-1)+1 evenly spaced
    points on [1/2, 1-delta]; the two lists share the point 1/2, kept once.
    """
    half = 2 ** (bits - 1)
    left = np.linspace(NF_DELTA, 0.5, half)
    right = np.linspace(0.5, 1.0 - NF_DELTA, half + 1)
    return np.concatenate([left, right[1:]])


def nf_table(bits: int) -> np.ndarray:
    """q_i = Phi^-1(p_i), normalised by the last quantile; exact zero at p = 1/2."""
    p = nf_probabilities(bits)
    q = ndtri(p)
    t = q / q[-1]
    t[2 ** (bits - 1) - 1] = 0.0
    return t


# ----------------------------------------------------------------------------
# quantise (Section 3, first equation; Section 4.2 for the absmax group scale)
# ----------------------------------------------------------------------------

def quantize(W, T_bits, group_size: int, dtype: str):
    """Q[n,k] = argmin_c |W[n,k]/s - T[c]| with s = absmax of the group (stored in dtype).

    Lowest index wins ties.  A group whose absmax is zero gets scale 0 and the
    index of the table's zero entry.  Returns (Q uint8 [N,K], S uint16 [N,K/B]).
    """
    W = np.asarray(W, dtype=np.float64)
    N, K = W.shape
    G = K // group_size
    T = to_f64(T_bits, dtype)
    Wg = W.reshape(N, G, group_size)
    # the stored scale is the 16-bit rounding of the group's absmax
    S_bits = from_f64(np.abs(Wg).max(axis=2), dtype)
    s = to_f64(S_bits, dtype)
    Q = np.empty((N, G, group_size), dtype=np.uint8)
    zero_idx = int(np.argmin(np.abs(T)))
    for n in range(N):
        for g in range(G):
            if s[n, g] == 0.0:
                Q[n, g, :] = zero_idx
                continue
            u = Wg[n, g] / s[n, g]
            Q[n, g, :] = np.argmin(np.abs(u[:, None] - T[None, :]), axis=1)
    return Q.reshape(N, K), S_bits


# ----------------------------------------------------------------------------
# packed layout (this project's definition; Section 3.1 gives the goal:
# weights reordered offline so that, once dequantised, they already sit in the
# matrix-unit operand order, and 3-bit weights split into a 2-bit and a 1-bit
# slice so that every load is a power-of-two number of bits)
# ----------------------------------------------------------------------------
# N is cut into row blocks of 16, K into tiles of TK (128 for 4-bit, 256 for 2- and 3-bit).
# Row blocks are grouped into super-blocks of SB consecutive row blocks: SB = 4 if N/16 is a multiple
# of 4 and not in the range 257..512, else 2 if N/16 is even, else 1.  Storage order: super-block, then K tile, then row block inside the
# super-block; tile (rb, kt) is tile number ((rb // SB) * (K/TK) + kt) * SB + rb % SB.  (So the SB
# tiles that cover 16*SB rows x TK columns are adjacent in memory.)  Inside a tile, "lane"
# l = 16*o + i (i = row inside the block, o = 0..3) owns, for each 32-wide K step t of the tile,
# the 8 consecutive indices
#       Q[16*rb + i, TK*kt + 32*t + 8*o + j],  j = 0..7.
#
# 4-bit: tile = 64 lanes x 16 B.  Lane l: four little-endian uint32 words d = 0..3
#        (d = step t); nibble j (bits 4j..4j+3) of word d = index j of step d.
# 2-bit: tile = 64 lanes x 16 B.  Lane l: words d = 0..3; 2-bit field e = 0..15
#        (bits 2e..2e+1) of word d = index j = e % 8 of step t = 2d + e // 8.
# 3-bit: tile = 1024 B "low" slice (index bits 0..1) + 512 B "high" slice (index bit 2).
#        low slice, lane l at 16*l: words d = 0..3; byte p = 0..3 of word d:
#            bits 0..1 = low2(index 2p   of step 2d),  bits 2..3 = low2(index 2p+1 of step 2d),
#            bits 4..5 = low2(index 2p   of step 2d+1), bits 6..7 = low2(index 2p+1 of step 2d+1).
#        high slice, lane l at 1024 + 8*l: words h = 0..1; byte p of word h:
#            bit 2u   = bit2(index 2p   of step 4h+u),
#            bit 2u+1 = bit2(index 2p+1 of step 4h+u),   u = 0..3.

TILE_K = {2: 256, 3: 256, 4: 128}


def packed_bytes(N: int, K: int, bits: int) -> int:
    return N * K * bits // 8


def super_block(N: int) -> int:
    """Row blocks per super-block: 4 if N/16 is a multiple of 4 and not in 257..512, else 2 if even, else 1."""
    nb = N // 16
    if nb % 4 == 0 and not (256 < nb <= 512):
        return 4
    return 2 if nb % 2 == 0 else 1


def _lane_view(Q: np.ndarray, bits: int) -> np.ndarray:
    """Q [N,K] -> A[tile, o, i, t, j] in storage order of the tiles;
    tile = ((rb // SB) * KT + kt) * SB + rb % SB holds Q[16rb+i, TK*kt + 32t + 8o + j]."""
    N, K = Q.shape
    TK = TILE_K[bits]
    if N % 16 or K % TK:
        raise ValueError("N must be a multiple of 16 and K of the tile width")
    SB = super_block(N)
    A = Q.reshape(N // 16 // SB, SB, 16, K // TK, TK // 32, 4, 8)   # sb, r, i, kt, t, o, j
    A = A.transpose(0, 3, 1, 5, 2, 4, 6)                             # sb, kt, r, o, i, t, j
    return A.reshape(N // 16, K // TK, 4, 16, TK // 32, 8)          # (sb,kt,r) flattened as [NB, KT]: storage order


def pack(Q, bits: int) -> np.ndarray:
    """Index matrix [N,K] (uint8, values < 2^bits) -> packed bytes (uint8, 1-D)."""
    Q = np.asarray(Q, dtype=np.uint8)
    if Q.size and int(Q.max()) >= (1 << bits):
        raise ValueError("index out of range")
    A = _lane_view(Q, bits).astype(np.uint32)
    NB, KT = A.shape[0], A.shape[1]
    if bits == 4:
        # word d = step d; nibble j
        sh = (4 * np.arange(8, dtype=np.uint32))
        words = (A << sh).sum(axis=5, dtype=np.uint32)                  # rb,kt,o,i,d
        return np.ascontiguousarray(words.astype("<u4")).view(np.uint8).reshape(-1)
    if bits == 2:
        # word d holds steps 2d, 2d+1; field e = 8*(t%2) + j
        B = A.reshape(NB, KT, 4, 16, 4, 2, 8)                            # rb,kt,o,i,d,t%2,j
        sh = (2 * (8 * np.arange(2, dtype=np.uint32)[:, None] + np.arange(8, dtype=np.uint32)[None, :]))
        words = (B << sh).sum(axis=(5, 6), dtype=np.uint32)             # rb,kt,o,i,d
        return np.ascontiguousarray(words.astype("<u4")).view(np.uint8).reshape(-1)
    if bits == 3:
        low2 = A & np.uint32(3)
        bit2 = A >> np.uint32(2)
        # low slice: word d, byte p, step parity s, pair member r: bit = 8p + 4s + 2r
        L = low2.reshape(NB, KT, 4, 16, 4, 2, 4, 2)                      # rb,kt,o,i,d,s,p,r
        p = np.arange(4, dtype=np.uint32)[None, :, None]
        s = np.arange(2, dtype=np.uint32)[:, None, None]
        r = np.arange(2, dtype=np.uint32)[None, None, :]
        lo_words = (L << (8 * p + 4 * s + 2 * r)).sum(axis=(5, 6, 7), dtype=np.uint32)   # rb,kt,o,i,d
        # high slice: word h, step-in-word u, byte p, member r: bit = 8p + 2u + r
        H = bit2.reshape(NB, KT, 4, 16, 2, 4, 4, 2)                      # rb,kt,o,i,h,u,p,r
        u = np.arange(4, dtype=np.uint32)[:, None, None]
        hi_words = (H << (8 * p + 2 * u + r)).sum(axis=(5, 6, 7), dtype=np.uint32)       # rb,kt,o,i,h
        lo_b = np.ascontiguousarray(lo_words.astype("<u4")).view(np.uint8).reshape(NB, KT, 1024)
        hi_b = np.ascontiguousarray(hi_words.astype("<u4")).view(np.uint8).reshape(NB, KT, 512)
        return np.concatenate([lo_b, hi_b], axis=2).reshape(-1)
    raise ValueError("bits must be 2, 3 or 4")


def unpack(packed, N: int, K: int, bits: int) -> np.ndarray:
    """Inverse of `pack`, written out per field with plain loops over the bit fields."""
    packed = np.asarray(packed, dtype=np.uint8).reshape(-1)
    if packed.size != packed_bytes(N, K, bits):
        raise ValueError("wrong packed size")
    TK = TILE_K[bits]
    NB, KT = N // 16, K // TK
    A = np.empty((NB, KT, 4, 16, TK // 32, 8), dtype=np.uint8)          # rb,kt,o,i,t,j
    if bits == 4:
        w = packed.view("<u4").reshape(NB, KT, 4, 16, 4)
        for d in range(4):
            for j in range(8):
                A[..., d, j] = (w[..., d] >> np.uint32(4 * j)) & np.uint32(15)
    elif bits == 2:
        w = packed.view("<u4").reshape(NB, KT, 4, 16, 4)
        for d in range(4):
            for e in range(16):
                A[..., 2 * d + e // 8, e % 8] = (w[..., d] >> np.uint32(2 * e)) & np.uint32(3)
    elif bits == 3:
        tiles = packed.reshape(NB, KT, 1536)
        lo = np.ascontiguousarray(tiles[:, :, :1024]).view("<u4").reshape(NB, KT, 4, 16, 4)
        hi = np.ascontiguousarray(tiles[:, :, 1024:]).view("<u4").reshape(NB, KT, 4, 16, 2)
        for t in range(8):
            for j in range(8):
                p, r = j // 2, j % 2
                low2 = (lo[..., t // 2] >> np.uint32(8 * p + 4 * (t % 2) + 2 * r)) & np.uint32(3)
                bit2 = (hi[..., t // 4] >> np.uint32(8 * p + 2 * (t % 4) + r)) & np.uint32(1)
                A[..., t, j] = low2 | (bit2 << np.uint32(2))
    else:
        raise ValueError("bits must be 2, 3 or 4")
    # A is in storage order (sb, kt, r) x (o, i, t, j); undo it: -> sb, r, i, kt, t, o, j
    SB = super_block(N)
    A = A.reshape(NB // SB, KT, SB, 4, 16, TK // 32, 8)
    return np.ascontiguousarray(A.transpose(0, 2, 4, 1, 5, 3, 6)).reshape(N, K)


# ----------------------------------------------------------------------------
# dequantise and matmul
# ----------------------------------------------------------------------------

def dequant(Q, T_bits, S_bits, group_size: int, dtype: str) -> np.ndarray:
    """W^[n,k] = round16( T[Q[n,k]] * S[n, k // B] ), returned as uint16 bit patterns [N,K]."""
    Q = np.asarray(Q)
    N, K = Q.shape
    T = to_f64(T_bits, dtype)
    S = to_f64(S_bits, dtype)
    if S.shape != (N, K // group_size):
        raise ValueError("scale shape must be [N, K / group_size]")
    prod = T[Q] * np.repeat(S, group_size, axis=1)
    return from_f64(prod, dtype)


def dequant_channel(Q, Tn_bits, S_bits, group_size: int, dtype: str) -> np.ndarray:
    """One table per output row (Section 2.3: lookup tables at the output-channel level):
    W^[n,k] = round16( T[n, Q[n,k]] * S[n, k // B] ), Tn_bits of shape [N, 2^b]."""
    Q = np.asarray(Q)
    N, K = Q.shape
    T = to_f64(Tn_bits, dtype)
    S = to_f64(S_bits, dtype)
    if T.shape[0] != N or S.shape != (N, K // group_size):
        raise ValueError("table shape must be [N, 2^b] and scale shape [N, K / group_size]")
    W = np.empty((N, K), dtype=np.float64)
    for n in range(N):
        W[n] = T[n][Q[n]]
    return from_f64(W * np.repeat(S, group_size, axis=1), dtype)


def dequant_vectors(V, C_bits, S_bits, group_size: int, dtype: str) -> np.ndarray:
    """Vector codebook (Section 5: vector codebooks as a further use of a lookup kernel): index V[n, j] selects the
    d adjacent weights d*j .. d*j + d - 1 from C, a table of vectors of shape [E, d]:
    W^[n, d*j + c] = round16( C[V[n, j], c] * S[n, d*j // B] ), c = 0 .. d-1 (d divides B: a vector lies in one group)."""
    V = np.asarray(V)
    N, Kd = V.shape
    C = to_f64(C_bits, dtype)
    S = to_f64(S_bits, dtype)
    if C.ndim != 2:
        raise ValueError("codebook shape must be [E, d]")
    d = C.shape[1]
    K = d * Kd
    if group_size % d or S.shape != (N, K // group_size):
        raise ValueError("d must divide the group, and the scale shape must be [N, K / group_size]")
    if V.min() < 0 or V.max() >= C.shape[0]:
        raise ValueError("codebook index out of range")
    W = C[V].reshape(N, K)                      # [N, K/d, d] -> [N, K]: a vector's values side by side
    return from_f64(W * np.repeat(S, group_size, axis=1), dtype)


def matmul_f64(X_bits, What_bits, dtype: str) -> np.ndarray:
    """Y[m,n] = sum_k X[m,k] * W^[n,k] in float64; not rounded."""
    X = to_f64(X_bits, dtype)
    W = to_f64(What_bits, dtype)
    return X @ W.T


def lut_matmul(X_bits, packed, S_bits, T_bits, bits: int, group_size: int,
               N: int, K: int, dtype: str) -> np.ndarray:
    """The whole path: unpack -> table lookup -> group scale -> fp64 matmul."""
    Q = unpack(packed, N, K, bits)
    What = dequant(Q, T_bits, S_bits, group_size, dtype)
    return matmul_f64(X_bits, What, dtype)


def rel_fro_err(Y, Y_ref) -> float:
    """||Y - Y_ref||_F / ||Y_ref||_F, both widened to float64."""
    Y = np.asarray(Y, dtype=np.float64)
    Y_ref = np.asarray(Y_ref, dtype=np.float64)
    den = float(np.linalg.norm(Y_ref))
    num = float(np.linalg.norm(Y - Y_ref))
    return num / den if den > 0 else num
