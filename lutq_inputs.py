"""Seeded synthetic inputs for the LUT-quantised matmul path.

This module only *makes inputs*: activations X, index matrices Q, group scales S
and lookup tables T, with the shapes and value distributions of the paper's
kernel benchmarks (Section 4.1: LLaMA-3-8B/70B layer shapes and N = K = 8192,
three random data sets per shape).  It contains nothing of the path under test:
no packing, no dequantisation, no matmul.  Both the CPU oracle's tests and the
HIP path's tests/benchmarks draw their inputs from here, so that the two sides
see identical bytes without sharing any of their own code.

All 16-bit floating-point tensors are carried as ``uint16`` bit patterns plus a
dtype tag (``"f16"`` or ``"bf16"``), because numpy has no bfloat16.

Input recipe (stands in for the paper's quantised LLaMA-3 weights, which need
model checkpoints that are not available):
  * X ~ N(0, 1), rounded to the 16-bit dtype.
  * W ~ N(0, 0.02^2) in fp32, cut into groups of ``group_size`` consecutive
    elements along K inside one output row.
  * ``lut="nf"``: table = NormalFloat-b (Section 4.2), scale = absmax of the
    group rounded to the 16-bit dtype, index = nearest table entry to W/scale
    (lowest index on ties).
  * ``lut="learned"``: table = 2^b sorted draws from N(0, 1) rounded to the
    dtype (an arbitrary "learned" table), scale = u * absmax with u ~ U(0.5, 2).
  * ``lut="random_index"``: indices uniform on {0..2^b-1} (worst case for
    lookup-table bank conflicts), NormalFloat table, scales ~ 0.02 * |N(0,1)| + 0.01.
"""
from __future__ import annotations

import dataclasses
import statistics

import numpy as np

DTYPES = ("f16", "bf16")


# ----------------------------------------------------------------------------
# 16-bit float encodings (format conversion only)
# ----------------------------------------------------------------------------
def encode16(x, dtype: str) -> np.ndarray:
    """Round float values to fp16 / bf16 (round-to-nearest-even), return uint16 bits."""
    x = np.asarray(x)
    if dtype == "f16":
        return np.ascontiguousarray(x.astype(np.float16)).view(np.uint16)
    if dtype == "bf16":
        u = np.ascontiguousarray(x.astype(np.float32)).view(np.uint32)
        lsb = (u >> np.uint32(16)) & np.uint32(1)
        r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
        return r.astype(np.uint16)
    raise ValueError(f"unknown dtype {dtype!r}")


def decode16(bits, dtype: str) -> np.ndarray:
    """uint16 bit patterns -> float32 values (exact)."""
    bits = np.ascontiguousarray(np.asarray(bits, dtype=np.uint16))
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float32)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    raise ValueError(f"unknown dtype {dtype!r}")


# ----------------------------------------------------------------------------
# tables
# ----------------------------------------------------------------------------
def normal_float_table(bits: int) -> np.ndarray:
    """NormalFloat-b table in float64 (recipe of Section 4.2).

    Probabilities: 2^(b-1) evenly spaced values on [delta, 1/2] followed by the
    2^(b-1)+1 evenly spaced values on [1/2, 1-delta] with the shared 1/2 counted
    once; Gaussian quantiles of those, divided by the last one; the entry at
    index 2^(b-1)-1 (probability 1/2) is an exact zero.
    """
    half = 1 << (bits - 1)
    delta = 0.5 * (1.0 / 30.0 + 1.0 / 32.0)
    lo = [delta + (0.5 - delta) * i / (half - 1) for i in range(half)] if half > 1 else [0.5]
    hi = [0.5 + (1.0 - delta - 0.5) * i / half for i in range(half + 1)]
    probs = lo + hi[1:]
    nd = statistics.NormalDist()
    q = np.array([nd.inv_cdf(p) for p in probs], dtype=np.float64)
    t = q / q[-1]
    t[half - 1] = 0.0
    return t


@dataclasses.dataclass
class Case:
    """One synthetic problem instance.  16-bit tensors are uint16 bit patterns."""
    M: int
    N: int
    K: int
    bits: int
    group_size: int
    dtype: str
    X: np.ndarray        # [M, K] uint16
    Q: np.ndarray        # [N, K] uint8, values < 2^bits
    S: np.ndarray        # [N, K // group_size] uint16
    T: np.ndarray        # [2^bits] uint16
    seed: int = 0
    lut: str = "nf"


def _nearest_index_sorted(u: np.ndarray, table32: np.ndarray) -> np.ndarray:
    """Index of the nearest entry of an ascending table; lowest index on ties."""
    mids = (table32[:-1].astype(np.float64) + table32[1:].astype(np.float64)) * 0.5
    return np.searchsorted(mids, u, side="left").astype(np.uint8)


def make_case(seed: int, M: int, N: int, K: int, bits: int, group_size: int,
              dtype: str = "f16", lut: str = "nf", x_std: float = 1.0) -> Case:
    assert dtype in DTYPES and bits in (2, 3, 4) and K % group_size == 0
    rng = np.random.Generator(np.random.PCG64(seed))
    G = K // group_size
    X = encode16(rng.standard_normal((M, K), dtype=np.float32) * np.float32(x_std), dtype)

    if lut == "random_index":
        T = encode16(normal_float_table(bits), dtype)
        Q = rng.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
        S = encode16(np.abs(rng.standard_normal((N, G), dtype=np.float32)) * np.float32(0.02)
                     + np.float32(0.01), dtype)
        return Case(M, N, K, bits, group_size, dtype, X, Q, S, T, seed, lut)

    if lut == "nf":
        T = encode16(normal_float_table(bits), dtype)
    elif lut == "learned":
        T = encode16(np.sort(rng.standard_normal(1 << bits)), dtype)
    else:
        raise ValueError(f"unknown lut kind {lut!r}")
    t32 = decode16(T, dtype)

    Q = np.empty((N, K), dtype=np.uint8)
    S = np.empty((N, G), dtype=np.uint16)
    zero_idx = int(np.argmin(np.abs(t32)))
    rows_per_chunk = max(1, (1 << 24) // K)
    for r0 in range(0, N, rows_per_chunk):
        r1 = min(N, r0 + rows_per_chunk)
        W = rng.standard_normal((r1 - r0, G, group_size), dtype=np.float32) * np.float32(0.02)
        absmax = np.abs(W).max(axis=2)
        if lut == "learned":
            absmax = absmax * rng.uniform(0.5, 2.0, size=absmax.shape).astype(np.float32)
        s16 = encode16(absmax, dtype)
        s32 = decode16(s16, dtype)
        with np.errstate(divide="ignore", invalid="ignore"):
            u = W / s32[:, :, None]
        q = _nearest_index_sorted(u.reshape(r1 - r0, K), t32)
        dead = np.repeat(s32 == 0, group_size, axis=1)
        q[dead] = zero_idx
        Q[r0:r1] = q
        S[r0:r1] = s16
    return Case(M, N, K, bits, group_size, dtype, X, Q, S, T, seed, lut)


# LLaMA-3 layer shapes (N, K) used by the paper's kernel benchmarks (Section 4.1).
LLAMA3_8B_SHAPES = {
    "qkv": (6144, 4096),
    "o": (4096, 4096),
    "gate_up": (28672, 4096),
    "down": (4096, 14336),
}
LLAMA3_70B_SHAPES = {
    "qkv": (10240, 8192),
    "o": (8192, 8192),
    "gate_up": (57344, 8192),
    "down": (8192, 28672),
}


def algorithmic_bytes(M: int, N: int, K: int, bits: int, group_size: int) -> int:
    """Bytes the method itself has to move per call: packed weights + scales + X + Y."""
    return N * K * bits // 8 + N * (K // group_size) * 2 + M * K * 2 + M * N * 2
