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
