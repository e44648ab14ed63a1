"""CPU oracle of the DIVISION activation codec -- TEST INFRASTRUCTURE ONLY.

Thin ctypes front end of ``division_oracle.c`` (plain scalar C written from the
paper: Sec. 4.1, Sec. 4.2, Eq. (quantization), Algorithm 1, Appendix D).  Only
the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the product never does, and nothing here touches the GPU
library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

F32 = 0
BF16 = 1
F32_C16 = 2      # x fp32; H^L, delta, Delta cached as bfloat16 (the paper's format)

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "division_oracle.c"
_LIB = _HERE / "liboracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (no FMA contraction, no fast-math)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
             "-Wall", "-Wextra", "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(str(_LIB))
        i64, sz, u64, u32, vp, ci = (ctypes.c_int64, ctypes.c_size_t, ctypes.c_uint64,
                                     ctypes.c_uint32, ctypes.c_void_p, ctypes.c_int)
        L.oracle_packed_bytes.restype = sz
        L.oracle_packed_bytes.argtypes = [i64, i64, i64, i64, ci, ci, ci]
        L.oracle_packed_layout.restype = ci
        L.oracle_packed_layout.argtypes = [i64, i64, i64, i64, ci, ci, ci] + [ctypes.POINTER(sz)] * 6
        L.oracle_packed_bytes_3d.restype = sz
        L.oracle_packed_bytes_3d.argtypes = [i64, i64, i64, i64, i64, ci, ci, ci]
        L.oracle_packed_layout_3d.restype = ci
        L.oracle_packed_layout_3d.argtypes = [i64, i64, i64, i64, i64, ci, ci, ci] + [ctypes.POINTER(sz)] * 6
        L.oracle_compress_3d.restype = ci
        L.oracle_compress_3d.argtypes = [vp, i64, i64, i64, i64, i64, ci, ci, ci, u64, vp, vp, vp, vp, ci]
        L.oracle_decompress_3d.restype = ci
        L.oracle_decompress_3d.argtypes = [vp, i64, i64, i64, i64, i64, ci, ci, ci, vp, ci]
        L.oracle_compress.restype = ci
        L.oracle_compress.argtypes = [vp, i64, i64, i64, i64, ci, ci, ci, u64, vp, vp, vp, vp, ci]
        L.oracle_decompress.restype = ci
        L.oracle_decompress.argtypes = [vp, i64, i64, i64, i64, ci, ci, ci, vp, ci]
        L.oracle_hash32.restype = u32
        L.oracle_hash32.argtypes = [u64, u32, u32]
        L.oracle_hash32_fill.restype = None
        L.oracle_hash32_fill.argtypes = [u64, u32, u32, sz, vp]
        L.oracle_rand16.restype = u32
        L.oracle_rand16.argtypes = [u64, u32, u32]
        L.oracle_plane_keys.restype = None
        L.oracle_plane_keys.argtypes = [u64, u32, ctypes.POINTER(u32), ctypes.POINTER(u32)]
        L.oracle_float_to_bf16.restype = ctypes.c_uint16
        L.oracle_float_to_bf16.argtypes = [ctypes.c_float]
        L.oracle_bf16_to_float.restype = ctypes.c_float
        L.oracle_bf16_to_float.argtypes = [ctypes.c_uint16]
        L.oracle_mask_bytes.restype = sz
        L.oracle_mask_bytes.argtypes = [i64]
        L.oracle_relu_forward.restype = ci
        L.oracle_relu_forward.argtypes = [vp, i64, ci, vp, vp]
        L.oracle_dropout_threshold.restype = u32
        L.oracle_dropout_threshold.argtypes = [ctypes.c_float]
        L.oracle_dropout_forward.restype = ci
        L.oracle_dropout_forward.argtypes = [vp, i64, ci, ctypes.c_float, u64, vp, vp]
        L.oracle_mask_backward.restype = ci
        L.oracle_mask_backward.argtypes = [vp, vp, i64, ci, vp]
        L.oracle_maxpool_forward.restype = ci
        L.oracle_maxpool_forward.argtypes = [vp, i64, i64, i64, i64, ci, ci, vp, vp]
        L.oracle_maxpool_backward.restype = ci
        L.oracle_maxpool_backward.argtypes = [vp, vp, i64, i64, i64, i64, ci, ci, vp]
        _lib = L
    return _lib


def _np_dtype(dt: int):
    """numpy type of x and of the reconstruction"""
    return np.uint16 if dt == BF16 else np.float32


def packed_bytes(N, C, H, W, B, b, dt=F32) -> int:
    return int(lib().oracle_packed_bytes(N, C, H, W, B, b, dt))


def packed_bytes_3d(N, C, D, H, W, B, b, dt=F32) -> int:
    """3-D maps of Appendix D: planes of D x H x W elements, blocks of B x B x B."""
    return int(lib().oracle_packed_bytes_3d(N, C, D, H, W, B, b, dt))


def packed_layout_3d(N, C, D, H, W, B, b, dt=F32) -> dict:
    vals = [ctypes.c_size_t() for _ in range(6)]
    rc = lib().oracle_packed_layout_3d(N, C, D, H, W, B, b, dt, *[ctypes.byref(v) for v in vals])
    if rc:
        raise ValueError("invalid codec arguments")
    k = ["codes_off", "codes_bytes", "meta_off", "meta_bytes", "lfc_off", "lfc_bytes"]
    return {n: int(v.value) for n, v in zip(k, vals)}


def packed_layout(N, C, H, W, B, b, dt=F32) -> dict:
    vals = [ctypes.c_size_t() for _ in range(6)]
    rc = lib().oracle_packed_layout(N, C, H, W, B, b, dt, *[ctypes.byref(v) for v in vals])
    if rc:
        raise ValueError("invalid codec arguments")
    k = ["codes_off", "codes_bytes", "meta_off", "meta_bytes", "lfc_off", "lfc_bytes"]
    return {n: int(v.value) for n, v in zip(k, vals)}


def compress(x: np.ndarray, B: int, b: int, seed: int, dt: int = F32, threads: int = 1,
             debug: bool = False):
    """x: (N,C,H,W) float32 array, or uint16 array holding bf16 bit patterns; a 5-D array
    (N,C,D,H,W) is a batch of 3-D maps (Appendix D).

    Returns the packed buffer (uint8 array); with ``debug`` also a dict with
    the per-element pre-round value t, the 16 random bits r and the residual h.
    """
    assert x.ndim in (4, 5) and x.dtype == _np_dtype(dt) and x.flags.c_contiguous
    if x.ndim == 5:
        return _compress_3d(x, B, b, seed, dt, threads, debug)
    N, C, H, W = x.shape
    nb = packed_bytes(N, C, H, W, B, b, dt)
    if nb == 0:
        raise ValueError("invalid codec arguments")
    out = np.empty(nb, dtype=np.uint8)
    t = r = h = None
    if debug:
        t = np.empty(x.shape, np.float32)
        r = np.empty(x.shape, np.uint16)
        h = np.empty(x.shape, np.float32)
    rc = lib().oracle_compress(
        x.ctypes.data, N, C, H, W, dt, B, b, seed & (2 ** 64 - 1), out.ctypes.data,
        t.ctypes.data if debug else None, r.ctypes.data if debug else None,
        h.ctypes.data if debug else None, threads)
    if rc:
        raise ValueError("oracle_compress rejected its arguments")
    return (out, {"t": t, "r": r, "h": h}) if debug else out


def _compress_3d(x, B, b, seed, dt, threads, debug):
    N, C, D, H, W = x.shape
    nb = packed_bytes_3d(N, C, D, H, W, B, b, dt)
    if nb == 0:
        raise ValueError("invalid codec arguments")
    out = np.empty(nb, dtype=np.uint8)
    t = r = h = None
    if debug:
        t = np.empty(x.shape, np.float32)
        r = np.empty(x.shape, np.uint16)
        h = np.empty(x.shape, np.float32)
    rc = lib().oracle_compress_3d(
        x.ctypes.data, N, C, D, H, W, dt, B, b, seed & (2 ** 64 - 1), out.ctypes.data,
        t.ctypes.data if debug else None, r.ctypes.data if debug else None,
        h.ctypes.data if debug else None, threads)
    if rc:
        raise ValueError("oracle_compress_3d rejected its arguments")
    return (out, {"t": t, "r": r, "h": h}) if debug else out


def decompress(packed: np.ndarray, shape, B: int, b: int, dt: int = F32, threads: int = 1) -> np.ndarray:
    if len(shape) == 5:
        N, C, D, H, W = shape
        assert packed.dtype == np.uint8 and packed.flags.c_contiguous
        assert packed.size >= packed_bytes_3d(N, C, D, H, W, B, b, dt)
        out = np.empty(shape, dtype=_np_dtype(dt))
        rc = lib().oracle_decompress_3d(packed.ctypes.data, N, C, D, H, W, dt, B, b, out.ctypes.data, threads)
        if rc:
            raise ValueError("oracle_decompress_3d rejected its arguments")
        return out
    N, C, H, W = shape
    assert packed.dtype == np.uint8 and packed.flags.c_contiguous
    assert packed.size >= packed_bytes(N, C, H, W, B, b, dt)
    out = np.empty(shape, dtype=_np_dtype(dt))
    rc = lib().oracle_decompress(packed.ctypes.data, N, C, H, W, dt, B, b, out.ctypes.data, threads)
    if rc:
        raise ValueError("oracle_decompress rejected its arguments")
    return out


def split_packed(packed: np.ndarray, shape, B: int, b: int, dt: int = F32) -> dict:
    """Views of the three regions: codes u32[P][WPP], meta [P][2] (float32, or bf16 bit patterns as
    uint16 in the F32_C16 mode), lfc [P][LH][LW] (float32 for F32, else bf16 bit patterns)."""
    if len(shape) == 5:
        N, C, D, H, W = shape
        lay = packed_layout_3d(N, C, D, H, W, B, b, dt)
        P = N * C
        codes = packed[lay["codes_off"]:lay["codes_off"] + lay["codes_bytes"]].view(np.uint32).reshape(P, -1)
        meta = packed[lay["meta_off"]:lay["meta_off"] + lay["meta_bytes"]]
        meta = (meta.view(np.uint16) if dt == F32_C16 else meta.view(np.float32)).reshape(P, 2)
        lfc = packed[lay["lfc_off"]:lay["lfc_off"] + lay["lfc_bytes"]]
        lfc = (lfc.view(np.float32) if dt == F32 else lfc.view(np.uint16)).reshape(P, -(-D // B), -(-H // B), -(-W // B))
        return {"codes": codes, "meta": meta, "lfc": lfc}
    N, C, H, W = shape
    lay = packed_layout(N, C, H, W, B, b, dt)
    P = N * C
    LH, LW = -(-H // B), -(-W // B)
    codes = packed[lay["codes_off"]:lay["codes_off"] + lay["codes_bytes"]].view(np.uint32).reshape(P, -1)
    meta = packed[lay["meta_off"]:lay["meta_off"] + lay["meta_bytes"]]
    meta = (meta.view(np.uint16) if dt == F32_C16 else meta.view(np.float32)).reshape(P, 2)
    lfc = packed[lay["lfc_off"]:lay["lfc_off"] + lay["lfc_bytes"]]
    lfc = (lfc.view(np.float32) if dt == F32 else lfc.view(np.uint16)).reshape(P, LH, LW)
    return {"codes": codes, "meta": meta, "lfc": lfc}


def unpack_codes(codes: np.ndarray, HW: int, b: int) -> np.ndarray:
    """codes u32[P][WPP] -> uint8[P][HW] (element i in word i // (32/b), bit (i % (32/b)) * b)."""
    cpw = 32 // b
    P = codes.shape[0]
    shifts = (np.arange(cpw, dtype=np.uint32) * b)
    q = (codes[:, :, None] >> shifts[None, None, :]) & np.uint32((1 << b) - 1)
    return q.reshape(P, -1)[:, :HW].astype(np.uint8)


def hash32(seed: int, plane: int, j: int) -> int:
    return int(lib().oracle_hash32(seed & (2 ** 64 - 1), plane, j))


def hash32_fill(seed: int, plane: int, j0: int, n: int) -> np.ndarray:
    out = np.empty(n, np.uint32)
    lib().oracle_hash32_fill(seed & (2 ** 64 - 1), plane, j0, n, out.ctypes.data)
    return out


def rand16(seed: int, plane: int, i: int) -> int:
    return int(lib().oracle_rand16(seed & (2 ** 64 - 1), plane, i))


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    return ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)


def bf16_to_f32(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32)


# ---------------------------------------------------------------- 1-bit masks (Relu / Dropout operators)

def mask_bytes(n: int) -> int:
    return int(lib().oracle_mask_bytes(n))


def relu_forward(x: np.ndarray, dt: int = F32):
    """x: flat or n-d array (float32, or uint16 bf16 bit patterns).  Returns (out, mask words)."""
    x = np.ascontiguousarray(x, dtype=_np_dtype(dt))
    y = np.empty_like(x)
    mask = np.empty(mask_bytes(x.size) // 4, dtype=np.uint32)
    rc = lib().oracle_relu_forward(x.ctypes.data, x.size, dt, y.ctypes.data, mask.ctypes.data)
    if rc:
        raise ValueError("oracle_relu_forward failed")
    return y, mask


def dropout_threshold(p: float) -> int:
    return int(lib().oracle_dropout_threshold(p))


def dropout_forward(x: np.ndarray, p: float, seed: int, dt: int = F32):
    x = np.ascontiguousarray(x, dtype=_np_dtype(dt))
    y = np.empty_like(x)
    mask = np.empty(mask_bytes(x.size) // 4, dtype=np.uint32)
    rc = lib().oracle_dropout_forward(x.ctypes.data, x.size, dt, p, seed & (2 ** 64 - 1), y.ctypes.data, mask.ctypes.data)
    if rc:
        raise ValueError("oracle_dropout_forward failed")
    return y, mask


def mask_backward(mask: np.ndarray, grad_out: np.ndarray, dt: int = F32) -> np.ndarray:
    g = np.ascontiguousarray(grad_out, dtype=_np_dtype(dt))
    mask = np.ascontiguousarray(mask, dtype=np.uint32)
    assert mask.size * 4 == mask_bytes(g.size)
    out = np.empty_like(g)
    rc = lib().oracle_mask_backward(mask.ctypes.data, g.ctypes.data, g.size, dt, out.ctypes.data)
    if rc:
        raise ValueError("oracle_mask_backward failed")
    return out


def maxpool_forward(x: np.ndarray, k: int, dt: int = F32):
    """x: (N, C, H, W).  Returns (y of shape (N, C, H//k, W//k), mask words over the input)."""
    x = np.ascontiguousarray(x, dtype=_np_dtype(dt))
    N, C, H, W = x.shape
    y = np.empty((N, C, H // k, W // k), dtype=x.dtype)
    mask = np.empty(mask_bytes(x.size) // 4, dtype=np.uint32)
    rc = lib().oracle_maxpool_forward(x.ctypes.data, N, C, H, W, dt, k, y.ctypes.data, mask.ctypes.data)
    if rc:
        raise ValueError("oracle_maxpool_forward failed")
    return y, mask


def maxpool_backward(mask: np.ndarray, grad_out: np.ndarray, shape, k: int, dt: int = F32) -> np.ndarray:
    N, C, H, W = shape
    g = np.ascontiguousarray(grad_out, dtype=_np_dtype(dt))
    assert g.shape == (N, C, H // k, W // k)
    mask = np.ascontiguousarray(mask, dtype=np.uint32)
    out = np.empty(shape, dtype=g.dtype)
    rc = lib().oracle_maxpool_backward(mask.ctypes.data, g.ctypes.data, N, C, H, W, dt, k, out.ctypes.data)
    if rc:
        raise ValueError("oracle_maxpool_backward failed")
    return out
