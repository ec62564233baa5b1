"""ctypes binding for liblutq.so.  Names and argument order follow include/lutq.h."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTED_SYMBOLS = (
    "lutq_status_string", "lutq_packed_bytes", "lutq_pack", "lutq_unpack", "lutq_workspace_bytes",
    "lutq_plan_default", "lutq_plan_default_for", "lutq_plan_check", "lutq_pack_layout", "lutq_plan_table_set", "lutq_plan_table_lookup", "lutq_matmul", "lutq_matmul_plan", "lutq_matmul_static", "lutq_matmul_channel", "lutq_matmul_pairs", "lutq_matmul_quads", "lutq_tune", "lutq_tune_candidates", "lutq_quantize", "lutq_dequant",
    "lutq_calib_stream_read", "lutq_calib_copy", "lutq_calib_matmul_trace",
)

LUTQ_F16, LUTQ_BF16 = 0, 1


class LutqError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: lutq status {code} ({_status_string(code)})")
        self.code = code


class _CPlan(ctypes.Structure):
    _fields_ = [("row_blocks_per_wave", ctypes.c_int), ("grid", ctypes.c_int),
                ("waves_per_workgroup", ctypes.c_int), ("tiles_in_flight", ctypes.c_int),
                ("row_groups_per_workgroup", ctypes.c_int), ("scheduling", ctypes.c_int),
                ("tiles_per_item", ctypes.c_int)]


class _CLayout(ctypes.Structure):
    _fields_ = [("tile_k", ctypes.c_int), ("tile_bytes", ctypes.c_int), ("row_blocks_per_super_block", ctypes.c_int),
                ("row_blocks", ctypes.c_int64), ("k_tiles", ctypes.c_int64)]


class _CPlanEntry(ctypes.Structure):
    _fields_ = [("bits", ctypes.c_int), ("group_size", ctypes.c_int), ("dtype", ctypes.c_int),
                ("m_min", ctypes.c_int64), ("m_max", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("plan", _CPlan)]


@dataclass
class Plan:
    """Work decomposition knobs of lutq_matmul_plan; 0 = library default."""
    row_blocks_per_wave: int = 0
    grid: int = 0
    waves_per_workgroup: int = 0
    tiles_in_flight: int = 0
    row_groups_per_workgroup: int = 0
    scheduling: int = 0           # 0 library chooses, 1 static teams, 2 work queue (M <= 4), 3 row streaming
                                  # (row_blocks_per_wave = 4 or 8 row blocks side by side, whole row blocks per workgroup)
    tiles_per_item: int = 0

    def _c(self) -> _CPlan:
        return _CPlan(self.row_blocks_per_wave, self.grid, self.waves_per_workgroup, self.tiles_in_flight,
                      self.row_groups_per_workgroup, self.scheduling, self.tiles_per_item)


def lib_path() -> str:
    return os.path.join(_PKG_DIR, "liblutq.so")


def load_library():
    """Loads liblutq.so; raises if it has not been built (there is no other code path)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2407_10960_amd.build` "
                           "(there is no CPU or PyTorch fallback)")
    # PyTorch ships its own HIP runtime and owns the device memory and streams this library works on: it has to be in
    # the process first, so that liblutq.so binds to that runtime and not to a second copy of its own (a library loaded
    # before torch would query and launch through a runtime that torch's allocations do not belong to).
    import torch  # noqa: F401
    lib = ctypes.CDLL(path)
    vp, i64, ci, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    lib.lutq_status_string.restype = ctypes.c_char_p
    lib.lutq_status_string.argtypes = [ci]
    lib.lutq_packed_bytes.restype = sz
    lib.lutq_packed_bytes.argtypes = [i64, i64, ci, ci]
    lib.lutq_pack.restype = ci
    lib.lutq_pack.argtypes = [vp, i64, i64, ci, ci, vp]
    lib.lutq_unpack.restype = ci
    lib.lutq_unpack.argtypes = [vp, i64, i64, ci, ci, vp]
    lib.lutq_workspace_bytes.restype = sz
    lib.lutq_workspace_bytes.argtypes = [i64, i64, ci, ci]
    lib.lutq_plan_default.restype = ci
    lib.lutq_plan_default.argtypes = [ci, ci, i64, i64, i64, ci, ctypes.POINTER(_CPlan)]
    lib.lutq_plan_default_for.restype = ci
    lib.lutq_plan_default_for.argtypes = [ci, ci, i64, i64, i64, ci, ci, ctypes.POINTER(_CPlan)]
    lib.lutq_plan_check.restype = ci
    lib.lutq_plan_check.argtypes = [ci, ci, i64, i64, i64, ci, ci, ctypes.POINTER(_CPlan)]
    lib.lutq_pack_layout.restype = ci
    lib.lutq_pack_layout.argtypes = [i64, i64, ci, ci, ctypes.POINTER(_CLayout)]
    lib.lutq_plan_table_set.restype = ci
    lib.lutq_plan_table_set.argtypes = [ctypes.POINTER(_CPlanEntry), ci]
    lib.lutq_plan_table_lookup.restype = ci
    lib.lutq_plan_table_lookup.argtypes = [ci, ci, i64, i64, i64, ci, ctypes.POINTER(_CPlan)]
    lib.lutq_matmul.restype = ci
    lib.lutq_matmul.argtypes = [vp, vp, vp, vp, ci, ci, i64, i64, i64, ci, vp, vp, sz, vp]
    lib.lutq_matmul_plan.restype = ci
    lib.lutq_matmul_plan.argtypes = [vp, vp, vp, vp, ci, ci, i64, i64, i64, ci, vp, vp, sz, vp,
                                     ctypes.POINTER(_CPlan)]
    lib.lutq_matmul_static.restype = ci
    lib.lutq_matmul_static.argtypes = [vp, vp, vp, vp, ci, ci, i64, i64, i64, ci, vp, vp, ctypes.POINTER(_CPlan)]
    lib.lutq_matmul_pairs.restype = ci
    lib.lutq_matmul_pairs.argtypes = [vp, vp, vp, vp, ci, i64, i64, i64, ci, vp, vp, sz, vp]
    lib.lutq_matmul_quads.restype = ci
    lib.lutq_matmul_quads.argtypes = [vp, vp, vp, vp, ci, i64, i64, i64, ci, vp, vp, sz, vp]
    lib.lutq_matmul_channel.restype = ci
    lib.lutq_matmul_channel.argtypes = [vp, vp, vp, vp, ci, ci, i64, i64, i64, ci, vp, vp, sz, vp]
    lib.lutq_tune.restype = ci
    lib.lutq_tune.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ci, vp, ci, ci, i64, i64, i64, ci, vp, vp,
                              sz, vp, ci, ctypes.POINTER(_CPlan), ctypes.POINTER(ctypes.c_float)]
    lib.lutq_tune_candidates.restype = ci
    lib.lutq_tune_candidates.argtypes = [ci, ci, i64, i64, i64, ci, ctypes.POINTER(_CPlan), ci,
                                         ctypes.POINTER(ctypes.c_int)]
    lib.lutq_quantize.restype = ci
    lib.lutq_quantize.argtypes = [vp, ci, vp, ci, ci, i64, i64, ci, vp, vp, vp]
    lib.lutq_dequant.restype = ci
    lib.lutq_dequant.argtypes = [vp, vp, vp, ci, ci, i64, i64, ci, vp, vp]
    lib.lutq_calib_stream_read.restype = ci
    lib.lutq_calib_stream_read.argtypes = [vp, sz, ci, vp, vp]
    lib.lutq_calib_copy.restype = ci
    lib.lutq_calib_copy.argtypes = [vp, vp, sz, ci, vp]
    lib.lutq_calib_matmul_trace.restype = ci
    lib.lutq_calib_matmul_trace.argtypes = [vp, vp, vp, vp, ci, ci, i64, i64, i64, ci, vp, vp, sz, vp,
                                            ctypes.POINTER(_CPlan), vp, sz, ctypes.POINTER(ctypes.c_int)]
    _LIB = lib
    return lib


def _status_string(code: int) -> str:
    try:
        return load_library().lutq_status_string(code).decode()
    except Exception:  # pragma: no cover
        return "?"


def _check(code: int, what: str):
    if code != 0:
        raise LutqError(code, what)


# ------------------------------------------------------------------ host side (offline packer)
def lutq_packed_bytes(N: int, K: int, bits: int, group_size: int) -> int:
    return int(load_library().lutq_packed_bytes(N, K, bits, group_size))


def lutq_pack(indices, bits: int, group_size: int) -> np.ndarray:
    """indices: [N, K] uint8 (numpy, or anything np.asarray accepts) -> packed bytes (numpy uint8, 1-D)."""
    lib = load_library()
    idx = np.ascontiguousarray(np.asarray(indices, dtype=np.uint8))
    if idx.ndim != 2:
        raise ValueError("indices must be [N, K]")
    N, K = idx.shape
    nbytes = lib.lutq_packed_bytes(N, K, bits, group_size)
    out = np.empty(max(int(nbytes), 1), dtype=np.uint8)
    _check(lib.lutq_pack(idx.ctypes.data, N, K, bits, group_size, out.ctypes.data), "lutq_pack")
    return out[:nbytes]


def lutq_unpack(packed, N: int, K: int, bits: int, group_size: int) -> np.ndarray:
    lib = load_library()
    buf = np.ascontiguousarray(np.asarray(packed, dtype=np.uint8)).reshape(-1)
    if buf.size != lib.lutq_packed_bytes(N, K, bits, group_size):
        raise ValueError("packed buffer has the wrong size for (N, K, bits)")
    out = np.empty((N, K), dtype=np.uint8)
    _check(lib.lutq_unpack(buf.ctypes.data, N, K, bits, group_size, out.ctypes.data), "lutq_unpack")
    return out


# ------------------------------------------------------------------ device side
def lutq_workspace_bytes(N: int, K: int, bits: int, group_size: int) -> int:
    return int(load_library().lutq_workspace_bytes(N, K, bits, group_size))


def _torch():
    import torch
    return torch


def _dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.float16:
        return LUTQ_F16
    if t.dtype == torch.bfloat16:
        return LUTQ_BF16
    raise TypeError("X, scales, lut and Y must be float16 or bfloat16")


def _stream_ptr(stream) -> int:
    torch = _torch()
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def new_workspace(N: int, K: int, bits: int, group_size: int, device="cuda"):
    """A zero-filled device workspace for lutq_matmul (reusable across calls on one stream)."""
    torch = _torch()
    n = lutq_workspace_bytes(N, K, bits, group_size)
    if n == 0:
        raise ValueError("unsupported problem")
    return torch.zeros(n, dtype=torch.uint8, device=device)


def lutq_plan_default(bits: int, group_size: int, M: int, N: int, K: int, dtype_code: int = LUTQ_F16) -> Plan:
    cp = _CPlan()
    _check(load_library().lutq_plan_default(bits, group_size, M, N, K, dtype_code, ctypes.byref(cp)),
           "lutq_plan_default")
    return Plan(cp.row_blocks_per_wave, cp.grid, cp.waves_per_workgroup, cp.tiles_in_flight,
                cp.row_groups_per_workgroup, cp.scheduling, cp.tiles_per_item)


def lutq_plan_default_for(bits: int, group_size: int, M: int, N: int, K: int, dtype_code: int = LUTQ_F16,
                          compute_units: int = 256) -> Plan:
    """The default plan for a device with that many compute units (host logic, no device needed)."""
    cp = _CPlan()
    _check(load_library().lutq_plan_default_for(bits, group_size, M, N, K, dtype_code, compute_units, ctypes.byref(cp)),
           "lutq_plan_default_for")
    return Plan(cp.row_blocks_per_wave, cp.grid, cp.waves_per_workgroup, cp.tiles_in_flight,
                cp.row_groups_per_workgroup, cp.scheduling, cp.tiles_per_item)


def lutq_plan_check(bits: int, group_size: int, M: int, N: int, K: int, dtype_code: int = LUTQ_F16,
                    compute_units: int = 256, plan: Plan | None = None) -> int:
    """Status code lutq_matmul_plan would give this plan (None = default) on such a device; 0 = accepted."""
    cp = plan._c() if plan is not None else None
    return int(load_library().lutq_plan_check(bits, group_size, M, N, K, dtype_code, compute_units,
                                              ctypes.byref(cp) if cp is not None else None))


def lutq_pack_layout(N: int, K: int, bits: int, group_size: int) -> dict:
    """Geometry of the packed form: tile_k, tile_bytes, row_blocks_per_super_block, row_blocks, k_tiles."""
    c = _CLayout()
    _check(load_library().lutq_pack_layout(N, K, bits, group_size, ctypes.byref(c)), "lutq_pack_layout")
    return {f: int(getattr(c, f)) for f, _ in _CLayout._fields_}


def lutq_plan_table_set(entries) -> None:
    """entries: iterable of (bits, group_size, dtype_code, m_min, m_max, N, K, Plan); replaces the table."""
    entries = list(entries)
    arr = (_CPlanEntry * max(len(entries), 1))()
    for i, (bits, group, dt, m0, m1, N, K, plan) in enumerate(entries):
        arr[i] = _CPlanEntry(bits, group, dt, m0, m1, N, K, plan._c())
    _check(load_library().lutq_plan_table_set(arr, len(entries)), "lutq_plan_table_set")


def lutq_plan_table_lookup(bits: int, group_size: int, M: int, N: int, K: int, dtype_code: int = LUTQ_F16):
    """The registered plan for this call, or None."""
    cp = _CPlan()
    code = load_library().lutq_plan_table_lookup(bits, group_size, M, N, K, dtype_code, ctypes.byref(cp))
    if code != 0:
        return None
    return Plan(cp.row_blocks_per_wave, cp.grid, cp.waves_per_workgroup, cp.tiles_in_flight,
                cp.row_groups_per_workgroup, cp.scheduling, cp.tiles_per_item)


def lutq_matmul(X, packed, scales, lut, bits: int, group_size: int, Y, workspace, stream=None,
                plan: Plan | None = None):
    """Y[M,N] = X[M,K] @ dequant(packed, scales, lut)^T on the GPU.  All tensors are caller-owned
    torch CUDA tensors (X/scales/lut/Y float16 or bfloat16, packed/workspace uint8)."""
    lib = load_library()
    if not (X.is_cuda and packed.is_cuda and scales.is_cuda and lut.is_cuda and Y.is_cuda and workspace.is_cuda):
        raise ValueError("lutq_matmul needs CUDA (HIP) tensors")
    for t in (X, packed, scales, lut, Y, workspace):
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous")
    code = _dtype_code(X)
    if not (_dtype_code(scales) == code and _dtype_code(lut) == code and _dtype_code(Y) == code):
        raise TypeError("X, scales, lut and Y must share one dtype")
    M, K = X.shape
    N = scales.shape[0]
    if scales.shape[1] * group_size != K or tuple(Y.shape) != (M, N) or lut.numel() != (1 << bits):
        raise ValueError("inconsistent shapes")
    if packed.numel() != lib.lutq_packed_bytes(N, K, bits, group_size):
        raise ValueError("packed buffer has the wrong size for (N, K, bits)")
    args = [X.data_ptr(), packed.data_ptr(), scales.data_ptr(), lut.data_ptr(), bits, group_size, M, N, K, code,
            Y.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr(stream)]
    if plan is None:
        _check(lib.lutq_matmul(*args), "lutq_matmul")
    else:
        cp = plan._c()
        _check(lib.lutq_matmul_plan(*args, ctypes.byref(cp)), "lutq_matmul_plan")
    return Y


STATIC_SCRATCH_BYTES = 64 * 1024 + 16 * 1024 * 1024


def lutq_matmul_static(X, packed, scales, lut, bits: int, group_size: int, Y, stream=None, plan: Plan | None = None):
    """lutq_matmul on the library's built-in scratch: no workspace argument, nothing is allocated."""
    lib = load_library()
    for t in (X, packed, scales, lut, Y):
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError("lutq_matmul_static needs contiguous CUDA (HIP) tensors")
    code = _dtype_code(X)
    if not (_dtype_code(scales) == code and _dtype_code(lut) == code and _dtype_code(Y) == code):
        raise TypeError("X, scales, lut and Y must share one dtype")
    M, K = X.shape
    N = scales.shape[0]
    if scales.shape[1] * group_size != K or tuple(Y.shape) != (M, N) or lut.numel() != (1 << bits):
        raise ValueError("inconsistent shapes")
    if packed.numel() != lib.lutq_packed_bytes(N, K, bits, group_size):
        raise ValueError("packed buffer has the wrong size for (N, K, bits)")
    cp = plan._c() if plan is not None else None
    _check(lib.lutq_matmul_static(X.data_ptr(), packed.data_ptr(), scales.data_ptr(), lut.data_ptr(), bits, group_size,
                                  M, N, K, code, Y.data_ptr(), _stream_ptr(stream),
                                  ctypes.byref(cp) if cp is not None else None), "lutq_matmul_static")
    return Y


def _matmul_codebook(name, dim, bits, X, packed, scales, codebook, group_size, Y, workspace, stream):
    lib = load_library()
    for t in (X, packed, scales, codebook, Y, workspace):
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError(f"{name} needs contiguous CUDA (HIP) tensors")
    code = _dtype_code(X)
    if not (_dtype_code(scales) == code and _dtype_code(codebook) == code and _dtype_code(Y) == code):
        raise TypeError("X, scales, codebook and Y must share one dtype")
    M, K = X.shape
    N = scales.shape[0]
    if scales.shape[1] * group_size != K or tuple(Y.shape) != (M, N) or tuple(codebook.shape) != (256, dim):
        raise ValueError("inconsistent shapes")
    if packed.numel() != lib.lutq_packed_bytes(N, K, bits, group_size):
        raise ValueError("packed buffer has the wrong size for (N, K)")
    _check(getattr(lib, name)(X.data_ptr(), packed.data_ptr(), scales.data_ptr(), codebook.data_ptr(), group_size,
                              M, N, K, code, Y.data_ptr(), workspace.data_ptr(),
                              workspace.numel() * workspace.element_size(), _stream_ptr(stream)), name)
    return Y


def lutq_matmul_pairs(X, packed, scales, codebook, group_size: int, Y, workspace, stream=None):
    """lutq_matmul with a codebook of 256 pairs of adjacent weights (one byte of the 4-bit layout = one index)."""
    return _matmul_codebook("lutq_matmul_pairs", 2, 4, X, packed, scales, codebook, group_size, Y, workspace, stream)


def lutq_matmul_quads(X, packed, scales, codebook, group_size: int, Y, workspace, stream=None):
    """lutq_matmul with a codebook of 256 quads of adjacent weights (one byte of the 2-bit layout = one index)."""
    return _matmul_codebook("lutq_matmul_quads", 4, 2, X, packed, scales, codebook, group_size, Y, workspace, stream)


def lutq_matmul_channel(X, packed, scales, luts, bits: int, group_size: int, Y, workspace, stream=None):
    """lutq_matmul with one table per output row: luts is [N, 2^bits]."""
    lib = load_library()
    for t in (X, packed, scales, luts, Y, workspace):
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError("lutq_matmul_channel needs contiguous CUDA (HIP) tensors")
    code = _dtype_code(X)
    if not (_dtype_code(scales) == code and _dtype_code(luts) == code and _dtype_code(Y) == code):
        raise TypeError("X, scales, luts and Y must share one dtype")
    M, K = X.shape
    N = scales.shape[0]
    if scales.shape[1] * group_size != K or tuple(Y.shape) != (M, N) or tuple(luts.shape) != (N, 1 << bits):
        raise ValueError("inconsistent shapes")
    if packed.numel() != lib.lutq_packed_bytes(N, K, bits, group_size):
        raise ValueError("packed buffer has the wrong size for (N, K, bits)")
    _check(lib.lutq_matmul_channel(X.data_ptr(), packed.data_ptr(), scales.data_ptr(), luts.data_ptr(), bits, group_size,
                                   M, N, K, code, Y.data_ptr(), workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), _stream_ptr(stream)), "lutq_matmul_channel")
    return Y


def lutq_tune_candidates(bits: int, group_size: int, M: int, N: int, K: int, dtype_code: int = LUTQ_F16) -> list:
    lib = load_library()
    n = ctypes.c_int(0)
    _check(lib.lutq_tune_candidates(bits, group_size, M, N, K, dtype_code, None, 0, ctypes.byref(n)),
           "lutq_tune_candidates")
    arr = (_CPlan * max(n.value, 1))()
    _check(lib.lutq_tune_candidates(bits, group_size, M, N, K, dtype_code, arr, n.value, ctypes.byref(n)),
           "lutq_tune_candidates")
    return [Plan(c.row_blocks_per_wave, c.grid, c.waves_per_workgroup, c.tiles_in_flight,
                 c.row_groups_per_workgroup, c.scheduling, c.tiles_per_item) for c in arr[:n.value]]


def lutq_tune(X, packed_ring, scales_ring, lut, bits: int, group_size: int, Y, workspace, stream=None,
              reps: int = 50):
    """Fastest plan for this problem by measurement: returns (Plan, microseconds per launch).
    packed_ring / scales_ring: lists of equally shaped weight sets visited in turn."""
    lib = load_library()
    if len(packed_ring) != len(scales_ring) or not packed_ring:
        raise ValueError("packed_ring and scales_ring must have the same, non-zero length")
    for t in (X, lut, Y, workspace, *packed_ring, *scales_ring):
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError("lutq_tune needs contiguous CUDA (HIP) tensors")
    code = _dtype_code(X)
    M, K = X.shape
    N = scales_ring[0].shape[0]
    if tuple(Y.shape) != (M, N) or lut.numel() != (1 << bits):
        raise ValueError("inconsistent shapes")
    for pk, sc in zip(packed_ring, scales_ring):
        if tuple(sc.shape) != (N, K // group_size) or _dtype_code(sc) != code:
            raise ValueError("inconsistent scales")
        if pk.numel() != lib.lutq_packed_bytes(N, K, bits, group_size):
            raise ValueError("packed buffer has the wrong size for (N, K, bits)")
    n = len(packed_ring)
    pk = (ctypes.c_void_p * n)(*[t.data_ptr() for t in packed_ring])
    sc = (ctypes.c_void_p * n)(*[t.data_ptr() for t in scales_ring])
    cp = _CPlan()
    us = ctypes.c_float(0.0)
    _check(lib.lutq_tune(X.data_ptr(), pk, sc, n, lut.data_ptr(), bits, group_size, M, N, K, code, Y.data_ptr(),
                         workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr(stream),
                         reps, ctypes.byref(cp), ctypes.byref(us)), "lutq_tune")
    return Plan(cp.row_blocks_per_wave, cp.grid, cp.waves_per_workgroup, cp.tiles_in_flight,
                cp.row_groups_per_workgroup, cp.scheduling, cp.tiles_per_item), us.value


def lutq_quantize(W, lut, bits: int, group_size: int, scales_out, packed_out, stream=None):
    """Quantises the dense device matrix W[N,K] (float32, or the 16-bit dtype of lut) against the table:
    writes the group scales and the packed indices that lutq_matmul consumes."""
    import torch
    lib = load_library()
    for t in (W, lut, scales_out, packed_out):
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError("lutq_quantize needs contiguous CUDA (HIP) tensors")
    code = _dtype_code(lut)
    w_f32 = W.dtype == torch.float32
    if not w_f32 and _dtype_code(W) != code:
        raise TypeError("W must be float32 or share the dtype of lut")
    if _dtype_code(scales_out) != code:
        raise TypeError("scales_out and lut must share one dtype")
    N, K = W.shape
    if tuple(scales_out.shape) != (N, K // group_size) or lut.numel() != (1 << bits):
        raise ValueError("inconsistent shapes")
    if packed_out.numel() * packed_out.element_size() != lib.lutq_packed_bytes(N, K, bits, group_size):
        raise ValueError("packed buffer has the wrong size for (N, K, bits)")
    _check(lib.lutq_quantize(W.data_ptr(), int(w_f32), lut.data_ptr(), bits, group_size, N, K, code,
                             scales_out.data_ptr(), packed_out.data_ptr(), _stream_ptr(stream)), "lutq_quantize")
    return scales_out, packed_out


def lutq_dequant(packed, scales, lut, bits: int, group_size: int, W_out, stream=None):
    """W_out[N,K] = round16(lut[Q] * scales) on the GPU (same lookup + scale routine as lutq_matmul)."""
    lib = load_library()
    code = _dtype_code(W_out)
    N, K = W_out.shape
    if not (packed.is_cuda and scales.is_cuda and lut.is_cuda and W_out.is_cuda):
        raise ValueError("lutq_dequant needs CUDA (HIP) tensors")
    for t in (packed, scales, lut, W_out):
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous")
    if not (_dtype_code(scales) == code and _dtype_code(lut) == code):
        raise TypeError("scales, lut and W_out must share one dtype")
    if scales.shape[0] != N or scales.shape[1] * group_size != K or lut.numel() != (1 << bits):
        raise ValueError("inconsistent shapes")
    if packed.numel() != lib.lutq_packed_bytes(N, K, bits, group_size):
        raise ValueError("packed buffer has the wrong size for (N, K, bits)")
    _check(lib.lutq_dequant(packed.data_ptr(), scales.data_ptr(), lut.data_ptr(), bits, group_size, N, K, code,
                            W_out.data_ptr(), _stream_ptr(stream)), "lutq_dequant")
    return W_out


# ------------------------------------------------------------------ measurement helpers
def calib_stream_read(src, grid: int, sink, stream=None):
    _check(load_library().lutq_calib_stream_read(src.data_ptr(), src.numel() * src.element_size(), grid,
                                                 sink.data_ptr(), _stream_ptr(stream)), "lutq_calib_stream_read")


def calib_copy(src, dst, grid: int, stream=None):
    _check(load_library().lutq_calib_copy(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(), grid,
                                          _stream_ptr(stream)), "lutq_calib_copy")


TRACE_STAMPS = ("start", "arguments arrived", "first loads issued", "table built", "first tile multiplied",
                "K loop done", "waves reduced", "outputs stored")


def calib_matmul_trace(X, packed, scales, lut, bits: int, group_size: int, Y, workspace, trace, stream=None,
                       plan: Plan | None = None) -> int:
    """One launch through the measurement build of the kernel; `trace` is an int64 CUDA tensor that
    receives [workgroup][16 wave slots][8] device timestamps (10 ns units).  Returns the number of
    workgroups launched."""
    lib = load_library()
    M, K = X.shape
    N = scales.shape[0]
    n = ctypes.c_int(0)
    cp = plan._c() if plan is not None else None
    _check(lib.lutq_calib_matmul_trace(X.data_ptr(), packed.data_ptr(), scales.data_ptr(), lut.data_ptr(), bits, group_size,
                                       M, N, K, _dtype_code(X), Y.data_ptr(), workspace.data_ptr(),
                                       workspace.numel() * workspace.element_size(), _stream_ptr(stream),
                                       ctypes.byref(cp) if cp is not None else None, trace.data_ptr(),
                                       trace.numel() * trace.element_size(), ctypes.byref(n)), "lutq_calib_matmul_trace")
    return n.value
