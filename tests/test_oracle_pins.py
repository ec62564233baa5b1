"""Pins for the CPU oracle: each check ties an oracle function to something other
than the oracle itself (exact rational arithmetic, closed forms, the forward
Gaussian CDF, structural invariants, brute force on tiny inputs).  The last test
plants plausible mistakes in the oracle and verifies that the pins notice.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

import lutq_inputs as gen
from oracle import lutq_oracle as orc

BITS = (2, 3, 4)
DTYPES = ("f16", "bf16")


# ----------------------------------------------------------------------------
# exact-rational helpers, independent of numpy's float conversions
# ----------------------------------------------------------------------------
def frac_of_bits(h: int, dtype: str) -> Fraction:
    """Decode an fp16 / bf16 bit pattern by the format's definition."""
    ebits, mbits = (5, 10) if dtype == "f16" else (8, 7)
    bias = (1 << (ebits - 1)) - 1
    sign = -1 if (h >> 15) & 1 else 1
    e = (h >> mbits) & ((1 << ebits) - 1)
    m = h & ((1 << mbits) - 1)
    assert e != (1 << ebits) - 1, "inf/nan not expected"
    if e == 0:
        return sign * Fraction(m, 1 << mbits) * Fraction(2) ** (1 - bias)
    return sign * (1 + Fraction(m, 1 << mbits)) * Fraction(2) ** (e - bias)


def round_frac_to_format(x: Fraction, dtype: str) -> Fraction:
    """Round-to-nearest-even of an exact rational onto the fp16 / bf16 grid."""
    ebits, mbits = (5, 10) if dtype == "f16" else (8, 7)
    bias = (1 << (ebits - 1)) - 1
    if x == 0:
        return Fraction(0)
    sign = -1 if x < 0 else 1
    a = abs(x)
    e = 0
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    while Fraction(2) ** e > a:
        e -= 1
    e = max(e, 1 - bias)                      # subnormal range shares the lowest exponent
    quantum = Fraction(2) ** (e - mbits)
    n = a / quantum
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return sign * fl * quantum


def rand16(rng, shape, dtype, scale=1.0):
    return gen.encode16(rng.standard_normal(shape).astype(np.float32) * np.float32(scale), dtype)


# ----------------------------------------------------------------------------
# pin 1: whole path against exact rational brute force on tiny inputs
# ----------------------------------------------------------------------------
def check_brute_force(o, bits, dtype, group, seed=0):
    rng = np.random.default_rng(seed)
    TK = 128 if bits == 4 else 256
    N, K, M = 16, TK, 3
    Q = rng.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    T = rand16(rng, (1 << bits,), dtype)
    S = rand16(rng, (N, K // group), dtype, 0.05)
    X = rand16(rng, (M, K), dtype)
    packed = o.pack(Q, bits)
    Y = o.lut_matmul(X, packed, S, T, bits, group, N, K, dtype)
    What = o.dequant(o.unpack(packed, N, K, bits), T, S, group, dtype)
    Tf = [frac_of_bits(int(t), dtype) for t in T]
    for n in range(N):
        w_row = []
        for k in range(K):
            w = round_frac_to_format(Tf[int(Q[n, k])] * frac_of_bits(int(S[n, k // group]), dtype), dtype)
            assert frac_of_bits(int(What[n, k]), dtype) == w, (n, k)
            w_row.append(w)
        for m in range(M):
            y = sum(frac_of_bits(int(X[m, k]), dtype) * w_row[k] for k in range(K))
            assert abs(float(y) - Y[m, n]) <= 1e-12 * max(1.0, abs(float(y))), (m, n)


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("dtype,group", [("f16", 32), ("f16", 128), ("bf16", 64)])
def test_brute_force_exact_rational(bits, dtype, group):
    check_brute_force(orc, bits, dtype, group)


def test_fraction_rounding_helper_matches_format_definition():
    # the helper itself: ties to even, subnormals, and identity on representable values
    assert round_frac_to_format(Fraction(2049, 1), "f16") == 2048          # tie -> even
    assert round_frac_to_format(Fraction(2051, 1), "f16") == 2052          # tie -> even (up)
    assert round_frac_to_format(Fraction(1, 2 ** 25), "f16") == 0          # half the least subnormal -> even (0)
    assert round_frac_to_format(Fraction(3, 2 ** 25), "f16") == Fraction(2, 2 ** 24)
    for h in (0x0001, 0x03FF, 0x0400, 0x3C00, 0x7BFF, 0xBC01):
        v = frac_of_bits(h, "f16")
        assert round_frac_to_format(v, "f16") == v
    assert frac_of_bits(0x3F80, "bf16") == 1 and frac_of_bits(0x3C00, "f16") == 1


# ----------------------------------------------------------------------------
# pin 2: one-hot activations read single dequantised weights back through the matmul
# ----------------------------------------------------------------------------
def check_one_hot_x(o, bits, dtype, group):
    rng = np.random.default_rng(1)
    TK = 128 if bits == 4 else 256
    N, K = 32, 2 * TK
    Q = rng.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    T = rand16(rng, (1 << bits,), dtype)
    S = rand16(rng, (N, K // group), dtype, 0.05)
    ks = rng.choice(K, size=8, replace=False)
    X = np.zeros((8, K), dtype=np.uint16)
    one = gen.encode16(np.array([1.0]), dtype)[0]
    X[np.arange(8), ks] = one
    Y = o.lut_matmul(X, o.pack(Q, bits), S, T, bits, group, N, K, dtype)
    for m, k in enumerate(ks):
        for n in range(N):
            w = round_frac_to_format(frac_of_bits(int(T[Q[n, k]]), dtype)
                                     * frac_of_bits(int(S[n, k // group]), dtype), dtype)
            assert Y[m, n] == float(w)


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("dtype,group", [("f16", 64), ("bf16", 32)])
def test_one_hot_x(bits, dtype, group):
    check_one_hot_x(orc, bits, dtype, group)


# ----------------------------------------------------------------------------
# pin 3: all-ones table isolates the scale indexing: Y = sum_g s[n,g] * sum_{k in g} x[m,k]
# ----------------------------------------------------------------------------
def check_all_ones_table(o, bits, group):
    dtype = "f16"
    rng = np.random.default_rng(2)
    TK = 128 if bits == 4 else 256
    N, K, M = 48, 2 * max(TK, group), 5
    Q = rng.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    T = gen.encode16(np.ones(1 << bits), dtype)
    S = rand16(rng, (N, K // group), dtype, 0.05)
    X = rand16(rng, (M, K), dtype)
    Y = o.lut_matmul(X, o.pack(Q, bits), S, T, bits, group, N, K, dtype)
    xs = gen.decode16(X, dtype).astype(np.float64).reshape(M, K // group, group).sum(axis=2)   # [M, G]
    ref = xs @ gen.decode16(S, dtype).astype(np.float64).T
    np.testing.assert_allclose(Y, ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("group", (32, 64, 128, 256))
def test_all_ones_table(bits, group):
    check_all_ones_table(orc, bits, group)


# ----------------------------------------------------------------------------
# pin 4: a uniform-integer table reproduces min-max int-b group quantisation (Section 2.3)
# ----------------------------------------------------------------------------
def check_uniform_integer_table(o, bits, group):
    dtype = "f16"
    rng = np.random.default_rng(3)
    TK = 128 if bits == 4 else 256
    N, K, M = 16, TK, 4
    W = rng.standard_normal((N, K)) * 0.02
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    Wg = W.reshape(N, K // group, group)
    # scales with a short significand so that s*q needs no rounding in fp16
    s = np.abs(Wg).max(axis=2) / max(hi, 1)
    s = gen.decode16(gen.encode16(s, dtype) & np.uint16(0xFFF0), dtype).astype(np.float64)
    q = np.clip(np.rint(Wg / s[:, :, None]), lo, hi).astype(np.int64)        # min-max quantiser
    T = gen.encode16(np.arange(lo, hi + 1, dtype=np.float64), dtype)
    Q = (q - lo).astype(np.uint8).reshape(N, K)
    S = gen.encode16(s, dtype)
    What = o.dequant(Q, T, S, group, dtype)
    ref = (s[:, :, None] * q).reshape(N, K)                                    # plain int-b dequantisation
    assert np.array_equal(gen.decode16(What, dtype).astype(np.float64), ref)
    X = rand16(rng, (M, K), dtype)
    Y = o.lut_matmul(X, o.pack(Q, bits), S, T, bits, group, N, K, dtype)
    np.testing.assert_allclose(Y, gen.decode16(X, dtype).astype(np.float64) @ ref.T, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("group", (32, 128))
def test_uniform_integer_table(bits, group):
    check_uniform_integer_table(orc, bits, group)


# ----------------------------------------------------------------------------
# pin 5: NormalFloat table (Section 4.2): forward CDF, invariants, nesting
# ----------------------------------------------------------------------------
def _phi(x: float) -> float:
    return 0.5 * math.erfc(-x / math.sqrt(2.0))


def check_nf_table(o, bits):
    delta = 0.5 * (1 / 30 + 1 / 32)
    t = o.nf_table(bits)
    n = 1 << bits
    half = n // 2
    assert t.shape == (n,)
    assert np.all(np.diff(t) > 0)
    assert abs(t[0] + 1.0) < 1e-14 and t[-1] == 1.0       # Phi^-1(delta) = -Phi^-1(1-delta) up to rounding
    assert list(o.from_f64(t[[0, -1]], "f16")) == [0xBC00, 0x3C00]
    assert list(o.from_f64(t[[0, -1]], "bf16")) == [0xBF80, 0x3F80]
    assert t[half - 1] == 0.0 and not np.signbit(t[half - 1])
    assert (t < 0).sum() == half - 1 and (t > 0).sum() == half
    # z = Phi^-1(1 - delta) found by bisection on the forward CDF only
    a, b = 0.0, 10.0
    for _ in range(200):
        mid = 0.5 * (a + b)
        a, b = (mid, b) if _phi(mid) < 1 - delta else (a, mid)
    z = 0.5 * (a + b)
    probs = [_phi(float(v) * z) for v in t]
    assert abs(probs[0] - delta) < 1e-12 and abs(probs[-1] - (1 - delta)) < 1e-12
    assert abs(probs[half - 1] - 0.5) < 1e-15
    left = np.diff(probs[:half])
    right = np.diff(probs[half - 1:])
    if half > 2:
        assert np.allclose(left, left[0], rtol=0, atol=1e-12)
    assert np.allclose(right, right[0], rtol=0, atol=1e-12)
    assert abs(right[0] - (0.5 - delta) / half) < 1e-12
    if half > 1:
        assert abs(left[0] - (0.5 - delta) / (half - 1)) < 1e-12
    # sigma = 1 / Phi^-1(1 - delta): the table holds quantiles of N(0, sigma^2)
    assert abs(1.0 / z - 0.541087061664) < 1e-9


@pytest.mark.parametrize("bits", BITS)
def test_nf_table(bits):
    check_nf_table(orc, bits)


def test_nf_tables_nest_and_match_generator():
    # the b-bit positive side samples [1/2, 1-delta] at 2^(b-1)+1 points: every other one of the (b+1)-bit side
    for b in (2, 3):
        small, big = orc.nf_table(b), orc.nf_table(b + 1)
        np.testing.assert_allclose(small[(1 << (b - 1)) - 1:], big[(1 << b) - 1::2], rtol=0, atol=1e-15)
    for b in BITS:
        # an independent inverse-CDF implementation (Python's statistics module)
        np.testing.assert_allclose(orc.nf_table(b), gen.normal_float_table(b), rtol=0, atol=1e-12)


def test_nf_golden_bits_regression():
    """Stored fp16 / bf16 bit patterns written by tests/golden/make_golden.py from the oracle
    (the paper prints the recipe, Section 4.2, not the values): a regression guard only."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "nf_tables.txt")
    seen = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, dtype, *vals = line.split()
        bits = int(name[2:])
        got = orc.from_f64(orc.nf_table(bits), dtype)
        assert [f"{int(v):04x}" for v in got] == vals
        seen += 1
    assert seen == 6


# ----------------------------------------------------------------------------
# pin 6: the packed layout is a bijection of index bits onto packed bits
# ----------------------------------------------------------------------------
def check_pack_bijection(o, bits):
    rng = np.random.default_rng(4)
    TK = 128 if bits == 4 else 256
    N, K = 32, 2 * TK
    Q = rng.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    P = o.pack(Q, bits)
    assert P.dtype == np.uint8 and P.size == N * K * bits // 8
    assert np.array_equal(o.unpack(P, N, K, bits), Q)
    seen = set()
    zero = np.zeros((N, K), dtype=np.uint8)
    assert not o.pack(zero, bits).any()
    positions = [(int(rng.integers(N)), int(rng.integers(K))) for _ in range(64)] + \
                [(0, 0), (N - 1, K - 1), (15, TK - 1), (16, TK)]
    for (n, k) in positions:
        for b in range(bits):
            Z = zero.copy()
            Z[n, k] = 1 << b
            bitsset = np.unpackbits(o.pack(Z, bits))
            assert bitsset.sum() == 1                       # one index bit -> exactly one packed bit
            pos = int(np.flatnonzero(bitsset)[0])
            seen.add(((n, k, b), pos))
    assert len({p for _, p in seen}) == len({s for s, _ in seen})   # distinct sources -> distinct bits
    full = np.full((N, K), (1 << bits) - 1, dtype=np.uint8)
    assert np.all(o.pack(full, bits) == 0xFF)
    # every lane's 8 consecutive indices of a 32-wide K step live in the same 16-byte lane slot (4-bit, 2-bit)
    if bits in (2, 4):
        Z = zero.copy()
        Z[5, 40:48] = (1 << bits) - 1                        # row 5, step 1, octet 1 -> lane 16*1+5
        nz = np.flatnonzero(o.pack(Z, bits))
        assert nz.min() // 16 == nz.max() // 16 == 16 * 1 + 5


@pytest.mark.parametrize("bits", BITS)
def test_pack_bijection(bits):
    check_pack_bijection(orc, bits)


def test_pack_rejects_bad_input():
    with pytest.raises(ValueError):
        orc.pack(np.full((16, 128), 16, dtype=np.uint8), 4)
    with pytest.raises(ValueError):
        orc.pack(np.zeros((8, 128), dtype=np.uint8), 4)
    with pytest.raises(ValueError):
        orc.pack(np.zeros((16, 128), dtype=np.uint8), 3)
    with pytest.raises(ValueError):
        orc.unpack(np.zeros(10, dtype=np.uint8), 16, 128, 4)


# ----------------------------------------------------------------------------
# pin 7: quantise = nearest table entry, absmax scale, lowest index on ties
# ----------------------------------------------------------------------------
def check_quantize(o, dtype):
    rng = np.random.default_rng(5)
    bits, group = 3, 32
    T = o.from_f64(o.nf_table(bits), dtype)
    W = (rng.standard_normal((4, 64)) * 0.02).astype(np.float32).astype(np.float64)
    W[1, 32:] = 0.0                                            # a dead group
    Q, S = o.quantize(W, T, group, dtype)
    s = gen.decode16(S, dtype).astype(np.float64)
    t = gen.decode16(T, dtype).astype(np.float64)
    assert np.array_equal(S, gen.encode16(np.abs(W.reshape(4, 2, 32)).max(axis=2), dtype))
    assert s[1, 1] == 0 and np.all(Q[1, 32:] == 3)
    for n in range(4):
        for k in range(64):
            sg = s[n, k // group]
            if sg == 0:
                continue
            d = [abs(Fraction(W[n, k]) / Fraction(sg) - Fraction(v)) for v in t]
            best = min(range(8), key=lambda c: (d[c], c))
            # float division may differ from the exact quotient only when two distances nearly tie
            assert Q[n, k] == best or abs(float(d[Q[n, k]] - d[best])) < 1e-12
    # exact tie: u exactly halfway between two entries -> the lower index
    T2 = gen.encode16(np.array([-1.0, 0.0, 0.5, 1.0]), dtype)
    W2 = np.zeros((1, 32)); W2[0, 0] = 1.0; W2[0, 1] = 0.25; W2[0, 2] = 0.75; W2[0, 3] = -0.5
    Q2, _ = o.quantize(W2, T2, 32, dtype)
    assert list(Q2[0, :4]) == [3, 1, 2, 0]


@pytest.mark.parametrize("dtype", DTYPES)
def test_quantize(dtype):
    check_quantize(orc, dtype)


def test_generator_matches_oracle_quantizer():
    """The input generator's fast quantiser follows the same definition as the oracle's."""
    for dtype in DTYPES:
        c = gen.make_case(7, 1, 16, 256, 4, 64, dtype, "nf")
        rng = np.random.Generator(np.random.PCG64(7))
        rng.standard_normal((1, 256), dtype=np.float32)
        W = rng.standard_normal((16, 4, 64), dtype=np.float32) * np.float32(0.02)
        Q, S = orc.quantize(W.reshape(16, 256).astype(np.float64), c.T, 64, dtype)
        assert np.array_equal(S, c.S)
        assert (Q != c.Q).mean() < 0.01          # fp32 vs fp64 division can flip near-ties only


# ----------------------------------------------------------------------------
# pin 8: 16-bit conversions against the exact-rational definition
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", DTYPES)
def test_conversions_exact(dtype):
    rng = np.random.default_rng(6)
    a = rand16(rng, (200,), dtype)
    b = rand16(rng, (200,), dtype, 0.01)
    prod = orc.to_f64(a, dtype) * orc.to_f64(b, dtype)
    got = orc.from_f64(prod, dtype)
    for i in range(200):
        fa, fb = frac_of_bits(int(a[i]), dtype), frac_of_bits(int(b[i]), dtype)
        assert Fraction(float(orc.to_f64(a[i:i + 1], dtype)[0])) == fa
        assert frac_of_bits(int(got[i]), dtype) == round_frac_to_format(fa * fb, dtype)
    if dtype == "f16":    # one product that lands in the subnormal range
        x = orc.from_f64(orc.to_f64(np.array([0x0400], np.uint16), dtype) * 0.5, dtype)
        assert x[0] == 0x0200
    if dtype == "bf16":   # general float64 inputs: ties to even, and a value just above a tie
        got = orc.from_f64(np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -40]), dtype)
        assert list(got) == [0x3F80, 0x3F82, 0x3F81]


def test_rel_fro_err():
    a = np.array([[3.0, 4.0]])
    assert orc.rel_fro_err(a, a) == 0.0
    assert abs(orc.rel_fro_err(a * 1.001, a) - 0.001) < 1e-12


# ----------------------------------------------------------------------------
# planted mistakes: every mutant must be caught by at least one pin
# ----------------------------------------------------------------------------
class _Mutant:
    """A copy of the oracle's namespace with one function replaced."""
    def __init__(self, **repl):
        self.__dict__.update({k: getattr(orc, k) for k in dir(orc) if not k.startswith("__")})
        self.__dict__.update(repl)
        # re-bind the composite entry point to the mutant's own parts
        def lut_matmul(X, packed, S, T, bits, group, N, K, dtype):
            Q = self.unpack(packed, N, K, bits)
            return self.matmul_f64(X, self.dequant(Q, T, S, group, dtype), dtype)
        self.lut_matmul = lut_matmul


def _mut_scale_mod(Q, T_bits, S_bits, group, dtype):
    N, K = Q.shape
    T, S = orc.to_f64(T_bits, dtype), orc.to_f64(S_bits, dtype)
    k = np.arange(K)
    return orc.from_f64(T[Q] * S[:, k % (K // group)], dtype)


def _mut_no_scale(Q, T_bits, S_bits, group, dtype):
    return orc.from_f64(orc.to_f64(T_bits, dtype)[Q], dtype)


def _mut_truncate(Q, T_bits, S_bits, group, dtype):
    T, S = orc.to_f64(T_bits, dtype), orc.to_f64(S_bits, dtype)
    prod = T[Q] * np.repeat(S, group, axis=1)
    bits = orc.from_f64(prod, dtype)
    over = np.abs(orc.to_f64(bits, dtype)) > np.abs(prod)
    return (bits - over.astype(np.uint16)).astype(np.uint16)      # round toward zero


def _mut_index_reversed(Q, T_bits, S_bits, group, dtype):
    return orc.dequant(Q, T_bits[::-1], S_bits, group, dtype)


def _mut_matmul_abs(X_bits, W_bits, dtype):
    return orc.to_f64(X_bits, dtype) @ np.abs(orc.to_f64(W_bits, dtype)).T


def _mut_unpack_swapped_pairs(packed, N, K, bits):
    Q = orc.unpack(packed, N, K, bits)
    return np.ascontiguousarray(Q.reshape(N, K // 2, 2)[:, :, ::-1]).reshape(N, K)


def _mut_nf_two_halves(bits):
    half = 2 ** (bits - 1)
    from scipy.special import ndtri
    p = np.concatenate([np.linspace(orc.NF_DELTA, 0.5, half + 1)[:-1], np.linspace(0.5, 1 - orc.NF_DELTA, half)])
    q = ndtri(p)
    t = q / q[-1]
    return t


MUTANTS = {
    "scale index k mod groups": dict(dequant=_mut_scale_mod),
    "scale dropped": dict(dequant=_mut_no_scale),
    "truncating rounding": dict(dequant=_mut_truncate),
    "table reversed": dict(dequant=_mut_index_reversed),
    "sign lost in matmul": dict(matmul_f64=_mut_matmul_abs),
    "pair members swapped in unpack": dict(unpack=_mut_unpack_swapped_pairs),
    "NF halves sized the other way round": dict(nf_table=_mut_nf_two_halves),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name):
    m = _Mutant(**MUTANTS[name])
    checks = [
        lambda: check_brute_force(m, 4, "f16", 32),
        lambda: check_brute_force(m, 3, "bf16", 64),
        lambda: check_one_hot_x(m, 2, "f16", 64),
        lambda: check_all_ones_table(m, 4, 32),
        lambda: check_uniform_integer_table(m, 3, 32),
        lambda: check_nf_table(m, 4),
        lambda: check_pack_bijection(m, 3),
    ]
    caught = 0
    for c in checks:
        try:
            c()
        except AssertionError:
            caught += 1
    assert caught >= 1, f"mutant '{name}' slipped through every pin"


# ----------------------------------------------------------------------------
# pin 9: one table per output row -- reduces to the shared-table path when all rows hold the same
# table, and matches an entry-by-entry exact-rational evaluation when they differ
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", DTYPES)
def test_channel_tables(dtype):
    rng = np.random.default_rng(11)
    bits, group, N, K = 3, 32, 5, 64
    Q = rng.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    S = rand16(rng, (N, K // group), dtype, 0.05)
    T = rand16(rng, (1 << bits,), dtype)
    same = np.tile(T, (N, 1))
    assert np.array_equal(orc.dequant_channel(Q, same, S, group, dtype), orc.dequant(Q, T, S, group, dtype))
    Tn = rand16(rng, (N, 1 << bits), dtype)
    W = orc.dequant_channel(Q, Tn, S, group, dtype)
    for n in range(N):
        for k in range(K):
            exact = frac_of_bits(int(Tn[n, Q[n, k]]), dtype) * frac_of_bits(int(S[n, k // group]), dtype)
            assert frac_of_bits(int(W[n, k]), dtype) == round_frac_to_format(exact, dtype), (n, k)
    with pytest.raises(ValueError):
        orc.dequant_channel(Q, Tn[:-1], S, group, dtype)


@pytest.mark.parametrize("dtype", ("f16", "bf16"))
@pytest.mark.parametrize("d", (2, 4))
def test_vector_codebook(dtype, d):
    """dequant_vectors against exact rationals element by element, and its reduction to the scalar table: a codebook
    whose entry e is (T[field 0 of e], T[field 1 of e], ...) with V = the d indices of a vector side by side in a
    byte (d = 2: nibbles, d = 4: bit pairs) is dequant itself."""
    rng = np.random.default_rng(12 + d)
    group, N, K = 32, 5, 128
    b = 8 // d                                    # bits per scalar index in the reduction
    V = rng.integers(0, 256, size=(N, K // d), dtype=np.uint8)
    S = rand16(rng, (N, K // group), dtype, 0.05)
    C = rand16(rng, (256, d), dtype)
    W = orc.dequant_vectors(V, C, S, group, dtype)
    assert W.shape == (N, K)
    for n in range(N):
        for k in range(K):
            exact = frac_of_bits(int(C[V[n, k // d], k % d]), dtype) * frac_of_bits(int(S[n, k // group]), dtype)
            assert frac_of_bits(int(W[n, k]), dtype) == round_frac_to_format(exact, dtype), (n, k)
    T = rand16(rng, (1 << b,), dtype)
    Q = rng.integers(0, 1 << b, size=(N, K), dtype=np.uint8)
    e = np.arange(256)
    Cs = np.stack([T[(e >> (b * c)) & ((1 << b) - 1)] for c in range(d)], axis=1)
    Vs = np.zeros((N, K // d), dtype=np.uint8)
    for c in range(d):
        Vs |= (Q[:, c::d] << (b * c)).astype(np.uint8)
    assert np.array_equal(orc.dequant_vectors(Vs, Cs, S, group, dtype), orc.dequant(Q, T, S, group, dtype))
    # a reversed vector is a different matrix
    assert not np.array_equal(orc.dequant_vectors(Vs, Cs[:, ::-1], S, group, dtype), orc.dequant(Q, T, S, group, dtype))
    with pytest.raises(ValueError):
        orc.dequant_vectors(V, C[:, :d - 1], S, group, dtype)
    with pytest.raises(ValueError):
        orc.dequant_vectors(V.astype(np.int32) + 1, C[:200], S, group, dtype)
