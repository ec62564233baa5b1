"""CPU-only tests of the boundary: the library loads and exports what include/*.h declares, the
offline packer (host code) matches the oracle's layout bit for bit, and argument validation returns
error codes before anything would be launched.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2407_10960_amd as lutq
from oracle import lutq_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = []
    for fn in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(lutq_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = lutq.load_library()
    declared = _declared_functions()
    assert len(declared) >= 11
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in include/ but not exported"
    assert set(lutq.EXPORTED_SYMBOLS) == set(declared)


@pytest.mark.parametrize("bits", (2, 3, 4))
@pytest.mark.parametrize("shape", [(16, 256), (48, 1024), (256, 768), (4096, 256), (4128, 256), (5120, 256), (8192, 256), (8224, 256)])
def test_pack_matches_oracle_layout_bit_exact(bits, shape):
    N, K = shape
    rng = np.random.default_rng(bits * 100 + N)
    for pattern in ("random", "zeros", "max", "walking"):
        if pattern == "random":
            Q = rng.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
        elif pattern == "zeros":
            Q = np.zeros((N, K), dtype=np.uint8)
        elif pattern == "max":
            Q = np.full((N, K), (1 << bits) - 1, dtype=np.uint8)
        else:
            Q = ((np.arange(N)[:, None] * 7 + np.arange(K)[None, :]) % (1 << bits)).astype(np.uint8)
        P = lutq.lutq_pack(Q, bits, 32)
        assert P.size == lutq.lutq_packed_bytes(N, K, bits, 32) == N * K * bits // 8
        assert np.array_equal(P, orc.pack(Q, bits))
        assert np.array_equal(lutq.lutq_unpack(P, N, K, bits, 32), Q)
        assert np.array_equal(orc.unpack(P, N, K, bits), Q)


@pytest.mark.parametrize("bits", (2, 3, 4))
def test_pack_single_hot_positions(bits):
    N, K = 32, 512
    rng = np.random.default_rng(11)
    for _ in range(20):
        n, k = int(rng.integers(N)), int(rng.integers(K))
        Q = np.zeros((N, K), dtype=np.uint8)
        Q[n, k] = (1 << bits) - 1
        P = lutq.lutq_pack(Q, bits, 64)
        assert np.array_equal(P, orc.pack(Q, bits))
        assert int(np.unpackbits(P).sum()) == bits


def test_pack_error_codes():
    lib = lutq.load_library()
    Q = np.zeros((16, 256), dtype=np.uint8)
    out = np.zeros(16 * 256, dtype=np.uint8)
    pk = lambda q, n, k, b, g, o: lib.lutq_pack(q, n, k, b, g, o)
    assert pk(None, 16, 256, 4, 128, out.ctypes.data) == 1
    assert pk(Q.ctypes.data, 16, 256, 4, 128, None) == 1
    assert pk(Q.ctypes.data, 16, 256, 5, 128, out.ctypes.data) == 2
    assert pk(Q.ctypes.data, 16, 256, 1, 128, out.ctypes.data) == 2
    assert pk(Q.ctypes.data, 16, 256, 4, 48, out.ctypes.data) == 3
    assert pk(Q.ctypes.data, 8, 256, 4, 128, out.ctypes.data) == 4
    assert pk(Q.ctypes.data, 16, 192, 4, 64, out.ctypes.data) == 4      # K not a multiple of the 4-bit tile
    assert pk(Q.ctypes.data, 16, 128, 3, 64, out.ctypes.data) == 4      # K not a multiple of the 3-bit tile
    bad = Q.copy(); bad[3, 7] = 8
    assert pk(bad.ctypes.data, 16, 256, 3, 128, out.ctypes.data) == 6
    assert pk(bad.ctypes.data, 16, 256, 4, 128, out.ctypes.data) == 0
    assert lutq.lutq_packed_bytes(16, 256, 7, 128) == 0
    assert lutq.lutq_packed_bytes(16, 100, 4, 128) == 0
    assert lutq.lutq_workspace_bytes(16, 100, 4, 128) == 0
    assert lutq.lutq_workspace_bytes(4096, 4096, 4, 128) > 0
    with pytest.raises(lutq.LutqError) as e:
        lutq.lutq_pack(bad, 2, 128)
    assert e.value.code == 6 and "index" in str(e.value)


def test_matmul_validation_returns_codes_before_any_launch():
    """Every one of these returns from host-side validation; no device call is made."""
    lib = lutq.load_library()
    buf = (ctypes.c_char * 4096)()
    base = ctypes.addressof(buf)
    a = (base + 15) & ~15                       # a 16-byte aligned fake pointer
    ws_bytes = lutq.lutq_workspace_bytes(16, 128, 4, 128)
    call = lambda X=a, P=a, S=a, T=a, bits=4, g=128, M=1, N=16, K=128, dt=0, Y=a, ws=a, wsb=ws_bytes: \
        lib.lutq_matmul(X, P, S, T, bits, g, M, N, K, dt, Y, ws, wsb, None)
    assert call(X=None) == 1 and call(P=None) == 1 and call(S=None) == 1 and call(T=None) == 1 and call(Y=None) == 1
    assert call(bits=5) == 2
    assert call(g=100) == 3
    assert call(g=64, K=128 + 32) == 4          # K not a tile multiple
    assert call(M=0) == 4 and call(M=129) == 4
    assert call(N=24) == 4
    assert call(dt=2) == 8
    assert call(X=a + 2) == 5 and call(Y=a + 8) == 5 and call(S=a + 4) == 5
    assert call(ws=None) == 7 and call(wsb=ws_bytes - 1) == 7
    dq = lib.lutq_dequant
    assert dq(None, a, a, 4, 128, 16, 128, 0, a, None) == 1
    assert dq(a, a, a, 9, 128, 16, 128, 0, a, None) == 2
    assert dq(a, a, a, 4, 128, 16, 128, 3, a, None) == 8
    assert dq(a, a, a, 4, 128, 16, 128, 0, a + 4, None) == 5
    assert lib.lutq_status_string(0) == b"ok" and b"workspace" in lib.lutq_status_string(7)


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    from paper_2407_10960_amd import binding
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "_PKG_DIR", str(tmp_path))
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        binding.lutq_pack(np.zeros((16, 128), dtype=np.uint8), 4, 128)


def test_product_never_imports_oracle():
    pkg = os.path.join(ROOT, "paper_2407_10960_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"


# ----------------------------------------------------------------------------
# host logic of the default work decomposition (no device needed)
# ----------------------------------------------------------------------------
def _sb(nb):
    return 4 if (nb % 4 == 0 and not (256 < nb <= 512)) else 2 if nb % 2 == 0 else 1


def test_default_plans_are_valid_for_random_problems():
    """Whatever the shape, the default plan respects the documented ranges and divisibility rules, for
    the 256 compute units of the target and for other device sizes."""
    rng = np.random.default_rng(3)
    for i in range(4000):
        bits = int(rng.choice([2, 3, 4]))
        tkb = 128 if bits == 4 else 256
        group = int(rng.choice([32, 64, 128, 256]))
        nb = int(rng.choice([1, 2, 3, 5, 8, 31, 64, 100, 255, 256, 257, 384, 448, 511, 512, 513, 640, 768, 1024, 1792, 3584,
                             4096, 5000, 9999, 16384]))
        kt = int(rng.integers(1, 300))
        K = tkb * kt
        if K % group:
            K *= 2
        M = int(rng.integers(1, 129))
        cus = int(rng.choice([256, 256, 256, 304, 64, 8, 1]))
        dt = int(rng.integers(0, 2))
        N = 16 * nb
        if N * K * bits // 8 >= 1 << 31:
            continue
        p = lutq.lutq_plan_default_for(bits, group, M, N, K, dt, cus)
        what = f"b{bits} g{group} M{M} N{N} K{K} cus{cus} dt{dt}: {p}"
        assert 4 <= p.waves_per_workgroup <= 16 and p.tiles_in_flight in (2, 4), what
        if p.scheduling == 3:                       # row streaming: M >= 5, whole row blocks per workgroup
            assert M >= 5 and p.row_blocks_per_wave in (4, 8) and p.tiles_in_flight == 2, what
            slices = 1
            if p.tiles_per_item:                    # K cut into slices across workgroups: one pass per share of row blocks
                assert M >= 9 and p.tiles_per_item * tkb >= 1792, what
                slices = -(-(K // tkb) // p.tiles_per_item)
                assert -(-(K // tkb) // slices) == p.tiles_per_item, what
                assert slices >= (3 if M > 24 or bits != 4 else 2) and p.grid % slices == 0 and cus // 2 <= p.grid <= cus, what
                assert p.row_groups_per_workgroup <= p.row_blocks_per_wave, what
            assert 1 <= p.grid // slices <= nb and p.row_groups_per_workgroup == nb // (p.grid // slices) <= 64, what
            assert (K // group * 2) % 16 == 0 or p.tiles_per_item or M > 32, what
            assert lutq.lutq_plan_check(bits, group, M, N, K, dt, cus) == 0, what
            if M <= 32:
                assert lutq.lutq_plan_check(bits, group, M, N, K, dt, cus, p) == 0, what
            continue
        assert p.row_blocks_per_wave in (1, 2, 4) and _sb(nb) % p.row_blocks_per_wave == 0, what
        nrg = nb // p.row_blocks_per_wave
        if p.scheduling == 2:                       # work queue: M <= 4, whole row groups per workgroup
            assert M <= 4 and p.row_blocks_per_wave <= 2 and 1 <= p.row_groups_per_workgroup <= 64, what
            assert p.row_groups_per_workgroup == nrg // p.grid and p.tiles_in_flight == 2, what
            assert p.tiles_per_item % 2 == 0 and (K // tkb) % p.tiles_per_item == 0, what
        else:
            assert p.scheduling == 1 and p.tiles_per_item == 0, what
            assert nrg % p.row_groups_per_workgroup == 0, what
            assert 1 <= p.row_groups_per_workgroup <= 16, what
            assert p.waves_per_workgroup % p.row_groups_per_workgroup == 0, what
            assert 1 <= p.grid and p.grid * p.row_groups_per_workgroup <= 4096, what
        # the library accepts its own default, given explicitly or not (kernel instance exists, LDS fits,
        # partial-sum slots suffice)
        assert lutq.lutq_plan_check(bits, group, M, N, K, dt, cus) == 0, what
        if M <= 32:                                 # (beyond 32 rows an explicit plan must also suit the last slice)
            assert lutq.lutq_plan_check(bits, group, M, N, K, dt, cus, p) == 0, what


def test_default_plans_of_the_llama3_shapes():
    """The measured choices for the benchmark's shapes on 256 compute units (4-bit, fp16, M = 1): a
    change here is a change of the benchmark's launch configuration."""
    want = {(6144, 4096, 128): (1, 256, 16, 2, 1, 2, 4), (4096, 4096, 128): (1, 256, 8, 2, 1, 2, 4),
            (28672, 4096, 128): (1, 256, 12, 2, 7, 2, 4), (4096, 14336, 128): (1, 256, 14, 2, 1, 1, 0),
            (10240, 8192, 64): (1, 256, 12, 2, 2, 2, 8), (8192, 8192, 64): (2, 256, 8, 2, 1, 1, 0),
            # the two largest: the work-queue kernel (one workgroup per compute unit, items of four K tiles)
            (57344, 8192, 64): (2, 256, 16, 2, 7, 2, 4), (8192, 28672, 64): (1, 256, 16, 2, 2, 2, 4)}
    for (N, K, g), plan in want.items():
        p = lutq.lutq_plan_default_for(4, g, 1, N, K, 0, 256)
        assert (p.row_blocks_per_wave, p.grid, p.waves_per_workgroup, p.tiles_in_flight, p.row_groups_per_workgroup,
                p.scheduling, p.tiles_per_item) == plan, (N, K, p)
    # beyond 32 rows: the one decomposition of the 64-row slices (4 bits, at least one row block per compute unit),
    # else the plan of the 32-row slices
    assert lutq.lutq_plan_default_for(4, 128, 100, 4096, 4096, 0, 256) == lutq.Plan(4, 256, 8, 2, 1, 3, 0)
    assert lutq.lutq_plan_default_for(4, 128, 40, 28672, 4096, 1, 256) == lutq.Plan(4, 256, 8, 2, 7, 3, 0)
    assert lutq.lutq_plan_default_for(4, 128, 100, 4096, 512, 0, 256).scheduling == 3          # scale rows of 8 bytes
    for (b, N, K) in [(3, 4096, 4096), (4, 2048, 4096)]:
        assert lutq.lutq_plan_default_for(b, 128, 100, N, K, 0, 256) == lutq.lutq_plan_default_for(b, 128, 32, N, K, 0, 256)
        assert lutq.lutq_plan_check(b, 128, 100, N, K, 0, 256, None) == 0
    with pytest.raises(lutq.LutqError):
        lutq.lutq_plan_default_for(4, 128, 1, 4096, 4096, 0, 0)


def test_default_plans_fitted_by_measurement():
    """Default plans of settings whose rule was fitted from tuner timings on 256 compute units (one
    case per rule: packed activation loads for M = 5..8, the 2-/3-bit rules for M = 9..15, small row
    groups and long K from 17 rows up, pairs of row blocks, joined small workgroups, bf16 team
    thresholds).  A change here must come with new timings."""
    want = {
        (4, 128, 8, 4096, 14336, 0): (1, 256, 7, 2, 1),          # seven waves: sixteen tiles = two scale chunks each
        (3, 128, 8, 12288, 4096, 0): (4, 256, 12, 2, 3, 3),       # row streaming: three row blocks per compute unit at 3 bits
        (3, 128, 12, 4096, 11008, 0): (4, 256, 12, 2, 4, 3),
        (3, 64, 12, 10240, 8192, 0): (1, 256, 10, 2, 10),
        (2, 128, 12, 5120, 13824, 0): (4, 240, 12, 2, 4, 3),
        (3, 128, 32, 5120, 13824, 0): (4, 240, 8, 2, 4, 3),
        (4, 128, 32, 1024, 4096, 0): (1, 128, 4, 2, 1),
        (4, 128, 4, 5120, 13824, 0): (2, 160, 8, 2, 1),
        (4, 128, 2, 5120, 5120, 0): (1, 256, 16, 2, 1, 2),         # work queue, shares of one and two row blocks
        (2, 128, 1, 32000, 4096, 1): (1, 500, 8, 2, 4),
        (3, 128, 3, 22016, 4096, 0): (1, 688, 4, 2, 2),
        (4, 64, 32, 10240, 8192, 1): (1, 256, 8, 4, 8),
        # row streaming (scheduling 3): row blocks that do not divide over the compute units, and one pass of
        # five to eight row blocks per compute unit from nine rows up
        (4, 64, 16, 10240, 8192, 1): (4, 256, 12, 2, 2, 3),
        (4, 128, 16, 22016, 4096, 0): (8, 256, 12, 2, 5, 3),
        (3, 128, 16, 28672, 4096, 1): (8, 256, 8, 2, 7, 3),
        (3, 128, 24, 28672, 4096, 0): (1, 224, 16, 2, 8, 1),
        # K slices on the row-streaming kernel: at most one row block per compute unit, a long K, 17..32 rows
        (4, 128, 20, 4096, 14336, 1): (4, 256, 8, 2, 4, 3),
        (3, 128, 32, 4096, 14336, 0): (4, 256, 8, 2, 4, 3),
        (4, 128, 32, 2048, 14336, 0): (4, 256, 8, 2, 4, 3),
        (4, 128, 24, 3072, 12288, 0): (4, 240, 8, 2, 4, 3),
        (4, 128, 16, 4096, 14336, 0): (4, 256, 12, 2, 4, 3),       # ... twelve waves up to sixteen rows
        (3, 128, 12, 4096, 14336, 1): (4, 256, 8, 2, 4, 3),        # (the 3-bit bf16 instance holds eight waves)
        (4, 128, 9, 4096, 14336, 0): (4, 256, 12, 2, 4, 3),
        (2, 128, 24, 4096, 14336, 1): (4, 256, 8, 2, 4, 3),
        (4, 128, 24, 4096, 11008, 0): (4, 256, 8, 2, 4, 3),        # ... uneven slices (22, 22, 21, 21 tiles), scale rows of 172 bytes
        (4, 128, 32, 5120, 13824, 0): (4, 240, 8, 2, 4, 3),        # ... 80 shares x 3 slices
        (4, 128, 12, 4096, 6144, 0): (1, 256, 6, 2, 1),            # ... three slices up to sixteen rows only from 4096 columns each
        (4, 128, 24, 4096, 6144, 0): (4, 192, 8, 2, 4, 3),
        (4, 64, 20, 8192, 28672, 1): (4, 256, 8, 2, 4, 3),         # ... two slices up to 24 rows
        (4, 64, 32, 8192, 28672, 1): (1, 256, 8, 4, 8),
        (4, 64, 16, 2048, 8192, 1): (1, 256, 4, 2, 1),             # ... nor on half the compute units up to sixteen rows
        (4, 64, 24, 2048, 8192, 1): (4, 128, 8, 2, 4, 3),
        (4, 64, 16, 8192, 28672, 1): (4, 256, 12, 2, 4, 3),        # ... two slices of 112 tiles: two row blocks per unit, a long K
        (4, 64, 16, 8192, 8192, 1): (2, 256, 4, 2, 1),             # ... not with two slices of 32 tiles
        (3, 64, 16, 8192, 28672, 1): (1, 256, 16, 2, 8),           # ... nor at 3 bits
        (4, 128, 32, 4096, 4096, 0): (1, 256, 4, 2, 1),            # ... nor with fewer than four slices of fourteen tiles
        (4, 128, 8, 28672, 4096, 0): (4, 448, 4, 2, 1),
        (4, 128, 32, 28672, 4096, 0): (2, 224, 8, 2, 4),
        # work queue with twelve waves: seven row blocks per compute unit at 2 and 3 bits
        (3, 128, 1, 28672, 4096, 0): (1, 256, 12, 2, 7, 2),
        (2, 128, 4, 28672, 4096, 1): (1, 256, 12, 2, 7, 2),
        (4, 128, 16, 28672, 4096, 0): (8, 256, 12, 2, 7, 3),
        (4, 128, 32, 28672, 4096, 1): (8, 256, 8, 2, 7, 3),
        (4, 64, 32, 57344, 8192, 0): (2, 256, 14, 2, 7, 1),
    }
    for (bits, g, M, N, K, dt), plan in want.items():
        p = lutq.lutq_plan_default_for(bits, g, M, N, K, dt, 256)
        got = (p.row_blocks_per_wave, p.grid, p.waves_per_workgroup, p.tiles_in_flight, p.row_groups_per_workgroup, p.scheduling)
        assert got == (plan if len(plan) == 6 else plan + (1,)), (bits, g, M, N, K, dt, p)


def test_plan_check_matches_documented_rules():
    ok = lambda *a, **k: lutq.lutq_plan_check(*a, **k)
    assert ok(4, 128, 1, 4096, 4096, 0, 256, lutq.Plan(1, 256, 12, 2, 1)) == 0
    assert ok(4, 128, 1, 4096, 4096, 0, 256, lutq.Plan(0, 4097, 0)) == 10          # grid beyond the slots
    assert ok(4, 128, 1, 4096, 4096, 0, 256, lutq.Plan(0, 0, 17)) == 10            # more than 16 waves
    assert ok(4, 128, 1, 4096, 4096, 0, 256, lutq.Plan(1, 0, 8, 2, 3)) == 10       # waves not a multiple of the teams
    assert ok(4, 128, 32, 4096, 4096, 0, 256, lutq.Plan(1, 0, 16, 2, 1)) == 10     # no 16-wave instance for 32 rows
    assert ok(4, 128, 36, 4096, 4096, 0, 256, lutq.Plan(1, 0, 16, 2, 1)) == 10     # ... nor for the 32-row slice of 36
    assert ok(4, 128, 4, 4096, 4096, 0, 256, lutq.Plan(1, 0, 16, 2, 1)) == 0
    assert ok(4, 128, 1, 8192, 4096, 0, 256, lutq.Plan(4, 0, 4)) == 10             # R = 4 does not divide the super-block of 2
    assert ok(4, 100, 1, 4096, 4096, 0, 256) == 3 and ok(5, 128, 1, 4096, 4096, 0, 256) == 2
    assert ok(4, 128, 129, 4096, 4096, 0, 256) == 4 and ok(4, 128, 1, 4096, 4096, 0, 0) == 4


def test_pack_layout_query_matches_the_documented_rule():
    """lutq_pack_layout reports the geometry the header documents, including the super-block rule with
    its frozen 257..512 exception."""
    for N, K, bits in [(16, 256, 2), (4096, 4096, 4), (8192, 8192, 4), (8192, 8192, 3), (6144, 4096, 4), (4112, 512, 2), (57344, 8192, 3)]:
        lay = lutq.lutq_pack_layout(N, K, bits, 64)
        nb = N // 16
        assert lay["row_blocks"] == nb and lay["tile_k"] == (128 if bits == 4 else 256)
        assert lay["tile_bytes"] == (1536 if bits == 3 else 1024) and lay["k_tiles"] == K // lay["tile_k"]
        assert lay["row_blocks_per_super_block"] == _sb(nb)
        assert lay["row_blocks"] * lay["k_tiles"] * lay["tile_bytes"] == lutq.lutq_packed_bytes(N, K, bits, 64)
    assert lutq.lutq_pack_layout(8192, 8192, 4, 64)["row_blocks_per_super_block"] == 2        # N/16 = 512: the exception
    assert lutq.lutq_pack_layout(8208, 8192, 4, 64)["row_blocks_per_super_block"] == 1        # N/16 = 513
    with pytest.raises(lutq.LutqError):
        lutq.lutq_pack_layout(100, 4096, 4, 64)


def test_plan_table_set_and_lookup():
    """Registered plans (the output of lutq_tune kept for later calls) are found by bits, group, dtype, N, K and
    an M range; the first match wins; an empty table finds nothing."""
    try:
        a, b = lutq.Plan(1, 256, 12, 2, 1, 1, 0), lutq.Plan(2, 256, 16, 2, 7, 2, 8)
        lutq.lutq_plan_table_set([(4, 128, 0, 1, 4, 4096, 4096, a), (4, 64, 0, 1, 1, 57344, 8192, b), (4, 128, 0, 1, 32, 4096, 4096, b)])
        assert lutq.lutq_plan_table_lookup(4, 128, 1, 4096, 4096, 0) == a
        assert lutq.lutq_plan_table_lookup(4, 128, 4, 4096, 4096, 0) == a
        assert lutq.lutq_plan_table_lookup(4, 128, 5, 4096, 4096, 0) == b
        assert lutq.lutq_plan_table_lookup(4, 128, 33, 4096, 4096, 0) is None
        assert lutq.lutq_plan_table_lookup(4, 128, 1, 4096, 4096, 1) is None            # other dtype
        assert lutq.lutq_plan_table_lookup(3, 128, 1, 4096, 4096, 0) is None
        assert lutq.lutq_plan_table_lookup(4, 64, 1, 57344, 8192, 0) == b
        lutq.lutq_plan_table_set([])
        assert lutq.lutq_plan_table_lookup(4, 128, 1, 4096, 4096, 0) is None
    finally:
        lutq.lutq_plan_table_set([])
