"""Python binding of the C ABI declared in include/division.h.

Argument marshalling only: every step of the codec runs in the HIP library.
PyTorch supplies device memory and streams.  There is no CPU fallback: if
libdivision.so is missing, importing a function from here raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

DIVISION_F32 = 0
DIVISION_BF16 = 1
DIVISION_F32_C16 = 2      # fp32 maps; H^L, delta, Delta cached as bfloat16 (the paper's format)

ERRORS = {1: "DIVISION_EINVAL", 2: "DIVISION_ESIZE", 3: "DIVISION_EALIGN",
          4: "DIVISION_ERANGE", 5: "DIVISION_EHIP"}

_LIB_PATH = Path(__file__).resolve().parent / "libdivision.so"
_lib = None


class DivisionError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what} failed: {ERRORS.get(code, code)}")
        self.code = code


def lib() -> ctypes.CDLL:
    """Loads the built library; builds it first only if no build exists."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            from . import _build
            _build.build()
        L = ctypes.CDLL(str(_LIB_PATH))
        i64, sz, u64, vp, ci = ctypes.c_int64, ctypes.c_size_t, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_int
        L.division_abi_version.restype = ci
        L.division_abi_version.argtypes = []
        L.division_packed_bytes.restype = sz
        L.division_packed_bytes.argtypes = [i64, i64, i64, i64, ci, ci, ci]
        L.division_packed_layout.restype = ci
        L.division_packed_layout.argtypes = [i64, i64, i64, i64, ci, ci, ci] + [ctypes.POINTER(sz)] * 6
        L.division_compress.restype = ci
        L.division_compress.argtypes = [vp, i64, i64, i64, i64, ci, ci, ci, u64, vp, sz, vp]
        L.division_decompress.restype = ci
        L.division_decompress.argtypes = [vp, sz, i64, i64, i64, i64, ci, ci, ci, vp, vp]
        pp = ctypes.POINTER(vp)
        L.division_compress_batch.restype = ci
        L.division_compress_batch.argtypes = [ci, pp, pp, ctypes.POINTER(u64), i64, i64, i64, i64, ci, ci, ci, sz, vp]
        L.division_decompress_batch.restype = ci
        L.division_decompress_batch.argtypes = [ci, pp, pp, sz, i64, i64, i64, i64, ci, ci, ci, vp]
        L.division_mask_bytes.restype = sz
        L.division_mask_bytes.argtypes = [i64]
        L.division_relu_forward.restype = ci
        L.division_relu_forward.argtypes = [vp, i64, ci, vp, vp, sz, vp]
        L.division_dropout_forward.restype = ci
        L.division_dropout_forward.argtypes = [vp, i64, ci, ctypes.c_float, u64, vp, vp, sz, vp]
        L.division_mask_backward.restype = ci
        L.division_mask_backward.argtypes = [vp, sz, vp, i64, ci, vp, vp]
        L.division_maxpool_forward.restype = ci
        L.division_maxpool_forward.argtypes = [vp, i64, i64, i64, i64, ci, ci, vp, vp, sz, vp]
        L.division_maxpool_backward.restype = ci
        L.division_maxpool_backward.argtypes = [vp, sz, vp, i64, i64, i64, i64, ci, ci, vp, vp]
        L.division_kernel_name.restype = ci
        L.division_kernel_name.argtypes = [ci, vp, i64, i64, i64, i64, ci, ci, ci, ctypes.c_char_p, sz]
        L.division_relu_compress.restype = ci
        L.division_relu_compress.argtypes = [vp, i64, i64, i64, i64, ci, ci, ci, u64, vp, vp, sz, vp, sz, vp]
        L.division_relu_compress_fused.restype = ci
        L.division_relu_compress_fused.argtypes = [i64, i64, i64, i64, ci, ci, ci]
        L.division_compress_maps.restype = ci
        L.division_compress_maps.argtypes = [ci, vp, vp]
        L.division_decompress_maps.restype = ci
        L.division_decompress_maps.argtypes = [ci, vp, vp]
        L.division_packed_bytes_3d.restype = sz
        L.division_packed_bytes_3d.argtypes = [i64, i64, i64, i64, i64, ci, ci, ci]
        L.division_packed_layout_3d.restype = ci
        L.division_packed_layout_3d.argtypes = [i64, i64, i64, i64, i64, ci, ci, ci] + [ctypes.POINTER(sz)] * 6
        L.division_compress_3d.restype = ci
        L.division_compress_3d.argtypes = [vp, i64, i64, i64, i64, i64, ci, ci, ci, u64, vp, sz, vp]
        L.division_decompress_3d.restype = ci
        L.division_decompress_3d.argtypes = [vp, sz, i64, i64, i64, i64, i64, ci, ci, ci, vp, vp]
        L.division_kernel_name_3d.restype = ci
        L.division_kernel_name_3d.argtypes = [ci, vp, i64, i64, i64, i64, i64, ci, ci, ci, ctypes.c_char_p, sz]
        _lib = L
    return _lib


def _dt(t: torch.dtype, c16: bool = False) -> int:
    """c16: cache H^L, delta and Delta as bfloat16 (fp32 maps only; the paper's format)."""
    if t == torch.float32:
        return DIVISION_F32_C16 if c16 else DIVISION_F32
    if t == torch.bfloat16 and not c16:
        return DIVISION_BF16
    raise TypeError(f"unsupported dtype {t}" + (" with c16" if c16 else ""))


def _stream(stream) -> int:
    """The hipStream_t to launch on, as an integer: the given stream (a torch.cuda.Stream or a raw
    handle), else torch's current stream through its public accessor."""
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def division_packed_bytes(N: int, C: int, H: int, W: int, B: int, b: int, dtype=torch.float32, c16: bool = False) -> int:
    return int(lib().division_packed_bytes(N, C, H, W, B, b, _dt(dtype, c16)))


def division_packed_layout(N: int, C: int, H: int, W: int, B: int, b: int, dtype=torch.float32, c16: bool = False) -> dict:
    vals = [ctypes.c_size_t() for _ in range(6)]
    rc = lib().division_packed_layout(N, C, H, W, B, b, _dt(dtype, c16), *[ctypes.byref(v) for v in vals])
    if rc:
        raise DivisionError(rc, "division_packed_layout")
    names = ["codes_off", "codes_bytes", "meta_off", "meta_bytes", "lfc_off", "lfc_bytes"]
    return {n: int(v.value) for n, v in zip(names, vals)}


def division_compress(x: torch.Tensor, B: int, b: int, seed: int, packed: torch.Tensor | None = None,
                      stream=None, c16: bool = False) -> torch.Tensor:
    """x: contiguous NCHW device tensor (float32 or bfloat16).  Returns the packed uint8 buffer."""
    if x.dim() != 4 or not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous 4-d device tensor")
    N, C, H, W = x.shape
    need = division_packed_bytes(N, C, H, W, B, b, x.dtype, c16)
    if need == 0:
        raise DivisionError(1, "division_packed_bytes")
    if packed is None:
        packed = torch.empty(need, dtype=torch.uint8, device=x.device)
    rc = lib().division_compress(x.data_ptr(), N, C, H, W, _dt(x.dtype, c16), B, b, seed & (2 ** 64 - 1),
                                 packed.data_ptr(), packed.numel() * packed.element_size(), _stream(stream))
    if rc:
        raise DivisionError(rc, "division_compress")
    return packed


def division_decompress(packed: torch.Tensor, shape, B: int, b: int, dtype=torch.float32,
                        out: torch.Tensor | None = None, stream=None, c16: bool = False) -> torch.Tensor:
    N, C, H, W = shape
    if out is None:
        out = torch.empty(shape, dtype=dtype, device=packed.device)
    rc = lib().division_decompress(packed.data_ptr(), packed.numel() * packed.element_size(),
                                   N, C, H, W, _dt(dtype, c16), B, b, out.data_ptr(), _stream(stream))
    if rc:
        raise DivisionError(rc, "division_decompress")
    return out


def division_packed_bytes_3d(N: int, C: int, D: int, H: int, W: int, B: int, b: int, dtype=torch.float32,
                             c16: bool = False) -> int:
    return int(lib().division_packed_bytes_3d(N, C, D, H, W, B, b, _dt(dtype, c16)))


def division_packed_layout_3d(N: int, C: int, D: int, H: int, W: int, B: int, b: int, dtype=torch.float32,
                              c16: bool = False) -> dict:
    vals = [ctypes.c_size_t() for _ in range(6)]
    rc = lib().division_packed_layout_3d(N, C, D, H, W, B, b, _dt(dtype, c16), *[ctypes.byref(v) for v in vals])
    if rc:
        raise DivisionError(rc, "division_packed_layout_3d")
    names = ["codes_off", "codes_bytes", "meta_off", "meta_bytes", "lfc_off", "lfc_bytes"]
    return {n: int(v.value) for n, v in zip(names, vals)}


def division_compress_3d(x: torch.Tensor, B: int, b: int, seed: int, packed: torch.Tensor | None = None,
                         stream=None, c16: bool = False) -> torch.Tensor:
    """x: contiguous N x C x D x H x W device tensor (float32 or bfloat16).  Returns the packed uint8 buffer."""
    if x.dim() != 5 or not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous 5-d device tensor")
    N, C, D, H, W = x.shape
    need = division_packed_bytes_3d(N, C, D, H, W, B, b, x.dtype, c16)
    if need == 0:
        raise DivisionError(1, "division_packed_bytes_3d")
    if packed is None:
        packed = torch.empty(need, dtype=torch.uint8, device=x.device)
    rc = lib().division_compress_3d(x.data_ptr(), N, C, D, H, W, _dt(x.dtype, c16), B, b, seed & (2 ** 64 - 1),
                                    packed.data_ptr(), packed.numel() * packed.element_size(), _stream(stream))
    if rc:
        raise DivisionError(rc, "division_compress_3d")
    return packed


def division_decompress_3d(packed: torch.Tensor, shape, B: int, b: int, dtype=torch.float32,
                           out: torch.Tensor | None = None, stream=None, c16: bool = False) -> torch.Tensor:
    N, C, D, H, W = shape
    if out is None:
        out = torch.empty(shape, dtype=dtype, device=packed.device)
    rc = lib().division_decompress_3d(packed.data_ptr(), packed.numel() * packed.element_size(),
                                      N, C, D, H, W, _dt(dtype, c16), B, b, out.data_ptr(), _stream(stream))
    if rc:
        raise DivisionError(rc, "division_decompress_3d")
    return out


def division_kernel_name_3d(direction: int, shape, B: int, b: int, dtype=torch.float32, data_ptr: int = 0,
                            c16: bool = False) -> str:
    buf = ctypes.create_string_buffer(128)
    N, C, D, H, W = shape
    rc = lib().division_kernel_name_3d(direction, data_ptr or None, N, C, D, H, W, _dt(dtype, c16), B, b, buf, 128)
    if rc:
        raise DivisionError(rc, "division_kernel_name_3d")
    return buf.value.decode()


class _MapDesc(ctypes.Structure):
    """division_map of include/division.h"""
    _fields_ = [("x", ctypes.c_void_p), ("packed", ctypes.c_void_p), ("xhat", ctypes.c_void_p),
                ("packed_bytes", ctypes.c_size_t),
                ("N", ctypes.c_int64), ("C", ctypes.c_int64), ("D", ctypes.c_int64), ("H", ctypes.c_int64), ("W", ctypes.c_int64),
                ("dt", ctypes.c_int), ("B", ctypes.c_int), ("b", ctypes.c_int), ("seed", ctypes.c_uint64)]


def _dims5(shape):
    """(N, C, D, H, W) of a 4-d (D = 1) or 5-d shape"""
    if len(shape) == 4:
        return shape[0], shape[1], 1, shape[2], shape[3]
    if len(shape) == 5:
        return tuple(shape)
    raise ValueError("maps are 4-d (N, C, H, W) or 5-d (N, C, D, H, W)")


def _per_map(v, n):
    return list(v) if isinstance(v, (list, tuple)) else [v] * n


def division_compress_maps(xs, B, b, seeds, packed=None, stream=None, c16: bool = False):
    """One call for maps of any mix of shapes (the maps one forward pass caches).  xs: contiguous 4-d or
    5-d device tensors; B, b: one value or one per map; seeds: one per map.  Returns the packed buffers."""
    n = len(xs)
    Bs, bs = _per_map(B, n), _per_map(b, n)
    if len(seeds) != n or len(Bs) != n or len(bs) != n:
        raise ValueError("one seed (and block size, code width) per map")
    descs = (_MapDesc * max(n, 1))()
    made = []
    for i, x in enumerate(xs):
        if not x.is_cuda or not x.is_contiguous():
            raise ValueError("every map must be a contiguous device tensor")
        N, C, D, H, W = _dims5(x.shape)
        use16 = c16 and x.dtype == torch.float32
        need = int(lib().division_packed_bytes_3d(N, C, D, H, W, Bs[i], bs[i], _dt(x.dtype, use16)))
        if need == 0:
            raise DivisionError(1, "division_packed_bytes_3d")
        pk = packed[i] if packed is not None else torch.empty(need, dtype=torch.uint8, device=x.device)
        made.append(pk)
        descs[i] = _MapDesc(x.data_ptr(), pk.data_ptr(), None, pk.numel() * pk.element_size(), N, C, D, H, W,
                            _dt(x.dtype, use16), Bs[i], bs[i], seeds[i] & (2 ** 64 - 1))
    rc = lib().division_compress_maps(n, descs, _stream(stream))
    if rc:
        raise DivisionError(rc, "division_compress_maps")
    return made


def division_decompress_maps(packed, shapes, B, b, dtypes=torch.float32, out=None, stream=None, c16: bool = False):
    """The reverse of division_compress_maps: rebuilds every map of a backward pass in one call."""
    n = len(packed)
    Bs, bs, dts = _per_map(B, n), _per_map(b, n), _per_map(dtypes, n)
    if len(shapes) != n or len(Bs) != n or len(bs) != n or len(dts) != n:
        raise ValueError("one shape (and block size, code width, dtype) per map")
    descs = (_MapDesc * max(n, 1))()
    made = []
    for i, pk in enumerate(packed):
        N, C, D, H, W = _dims5(shapes[i])
        use16 = c16 and dts[i] == torch.float32
        y = out[i] if out is not None else torch.empty(tuple(shapes[i]), dtype=dts[i], device=pk.device)
        made.append(y)
        descs[i] = _MapDesc(None, pk.data_ptr(), y.data_ptr(), pk.numel() * pk.element_size(), N, C, D, H, W,
                            _dt(dts[i], use16), Bs[i], bs[i], 0)
    rc = lib().division_decompress_maps(n, descs, _stream(stream))
    if rc:
        raise DivisionError(rc, "division_decompress_maps")
    return made


def _ptr_array(tensors):
    return (ctypes.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def division_compress_batch(xs, B: int, b: int, seeds, packed=None, stream=None, c16: bool = False):
    """xs: contiguous NCHW device tensors of ONE shape and dtype; seeds: one per tensor.
    Returns the list of packed uint8 buffers (those given in `packed`, else new ones)."""
    xs = list(xs)
    seeds = list(seeds)
    if len(seeds) != len(xs):
        raise ValueError("one seed per tensor")
    if not xs:
        return []
    x0 = xs[0]
    for x in xs:
        if x.dim() != 4 or not x.is_cuda or not x.is_contiguous() or x.shape != x0.shape or x.dtype != x0.dtype:
            raise ValueError("xs must be contiguous 4-d device tensors of one shape and dtype")
    N, C, H, W = x0.shape
    need = division_packed_bytes(N, C, H, W, B, b, x0.dtype, c16)
    if need == 0:
        raise DivisionError(1, "division_packed_bytes")
    if packed is None:
        packed = [torch.empty(need, dtype=torch.uint8, device=x0.device) for _ in xs]
    packed = list(packed)
    if len(packed) != len(xs):
        raise ValueError("one packed buffer per tensor")
    cap = min(p.numel() * p.element_size() for p in packed)
    sd = (ctypes.c_uint64 * len(xs))(*[s & (2 ** 64 - 1) for s in seeds])
    rc = lib().division_compress_batch(len(xs), _ptr_array(xs), _ptr_array(packed), sd, N, C, H, W,
                                       _dt(x0.dtype, c16), B, b, cap, _stream(stream))
    if rc:
        raise DivisionError(rc, "division_compress_batch")
    return packed


def division_decompress_batch(packed, shape, B: int, b: int, dtype=torch.float32, out=None, stream=None,
                              c16: bool = False):
    """packed: buffers written by division_compress(_batch) for maps of `shape`.  Returns the list of maps."""
    packed = list(packed)
    if not packed:
        return []
    N, C, H, W = shape
    if out is None:
        out = [torch.empty(shape, dtype=dtype, device=packed[0].device) for _ in packed]
    out = list(out)
    if len(out) != len(packed):
        raise ValueError("one output per packed buffer")
    nbytes = min(p.numel() * p.element_size() for p in packed)
    rc = lib().division_decompress_batch(len(packed), _ptr_array(packed), _ptr_array(out), nbytes,
                                         N, C, H, W, _dt(dtype, c16), B, b, _stream(stream))
    if rc:
        raise DivisionError(rc, "division_decompress_batch")
    return out


def division_kernel_name(direction: int, shape, B: int, b: int, dtype=torch.float32, data_ptr: int = 0,
                         c16: bool = False) -> str:
    """Name of the kernel instance a call would launch (direction 0 = compress, 1 = decompress)."""
    buf = ctypes.create_string_buffer(128)
    N, C, H, W = shape
    rc = lib().division_kernel_name(direction, data_ptr or None, N, C, H, W, _dt(dtype, c16), B, b, buf, 128)
    if rc:
        raise DivisionError(rc, "division_kernel_name")
    return buf.value.decode()


# ---------------------------------------------------------------- 1-bit masks (Relu / Dropout operators)

def division_mask_bytes(n: int) -> int:
    return int(lib().division_mask_bytes(n))


def _flat_ok(t: torch.Tensor, what: str):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{what} must be a contiguous device tensor")


def division_relu_forward(x: torch.Tensor, out: torch.Tensor | None = None, mask: torch.Tensor | None = None, stream=None):
    """Returns (y, mask): y = x where x > 0 else +0; mask = one bit per element (int32 words)."""
    _flat_ok(x, "x")
    n = x.numel()
    if out is None:
        out = torch.empty_like(x)
    if mask is None:
        mask = torch.empty(division_mask_bytes(n) // 4, dtype=torch.int32, device=x.device)
    rc = lib().division_relu_forward(x.data_ptr(), n, _dt(x.dtype), out.data_ptr(), mask.data_ptr(),
                                     mask.numel() * mask.element_size(), _stream(stream))
    if rc:
        raise DivisionError(rc, "division_relu_forward")
    return out, mask


def division_relu_compress(x: torch.Tensor, B: int, b: int, seed: int, out: torch.Tensor | None = None,
                           mask: torch.Tensor | None = None, packed: torch.Tensor | None = None, stream=None,
                           c16: bool = False):
    """Relu and the compression of its output in one call (one kernel for the large maps).
    Returns (y, mask, packed)."""
    if x.dim() != 4 or not x.is_cuda or not x.is_contiguous():
        raise ValueError("x must be a contiguous 4-d device tensor")
    N, C, H, W = x.shape
    n = x.numel()
    if out is None:
        out = torch.empty_like(x)
    if mask is None:
        mask = torch.empty(division_mask_bytes(n) // 4, dtype=torch.int32, device=x.device)
    if packed is None:
        need = division_packed_bytes(N, C, H, W, B, b, x.dtype, c16)
        if need == 0:
            raise DivisionError(1, "division_packed_bytes")
        packed = torch.empty(need, dtype=torch.uint8, device=x.device)
    rc = lib().division_relu_compress(x.data_ptr(), N, C, H, W, _dt(x.dtype, c16), B, b, seed & (2 ** 64 - 1),
                                      out.data_ptr(), mask.data_ptr(), mask.numel() * mask.element_size(),
                                      packed.data_ptr(), packed.numel() * packed.element_size(), _stream(stream))
    if rc:
        raise DivisionError(rc, "division_relu_compress")
    return out, mask, packed


def division_relu_compress_fused(shape, B: int, b: int, dtype=torch.float32, c16: bool = False) -> bool:
    N, C, H, W = shape
    return bool(lib().division_relu_compress_fused(N, C, H, W, _dt(dtype, c16), B, b))


def division_dropout_forward(x: torch.Tensor, p: float, seed: int, out: torch.Tensor | None = None,
                             mask: torch.Tensor | None = None, stream=None):
    """Returns (y, mask): y = x where the element is kept else +0 (no rescaling)."""
    _flat_ok(x, "x")
    n = x.numel()
    if out is None:
        out = torch.empty_like(x)
    if mask is None:
        mask = torch.empty(division_mask_bytes(n) // 4, dtype=torch.int32, device=x.device)
    rc = lib().division_dropout_forward(x.data_ptr(), n, _dt(x.dtype), p, seed & (2 ** 64 - 1), out.data_ptr(),
                                        mask.data_ptr(), mask.numel() * mask.element_size(), _stream(stream))
    if rc:
        raise DivisionError(rc, "division_dropout_forward")
    return out, mask


def division_mask_backward(mask: torch.Tensor, grad_out: torch.Tensor, out: torch.Tensor | None = None, stream=None):
    """grad_in = grad_out where the mask bit is set else +0."""
    _flat_ok(grad_out, "grad_out")
    if out is None:
        out = torch.empty_like(grad_out)
    rc = lib().division_mask_backward(mask.data_ptr(), mask.numel() * mask.element_size(), grad_out.data_ptr(),
                                      grad_out.numel(), _dt(grad_out.dtype), out.data_ptr(), _stream(stream))
    if rc:
        raise DivisionError(rc, "division_mask_backward")
    return out


def division_maxpool_forward(x: torch.Tensor, k: int, stream=None):
    """x: contiguous NCHW device tensor.  Returns (y of shape N x C x H//k x W//k, location mask over x)."""
    if x.dim() != 4:
        raise ValueError("x must be 4-d")
    _flat_ok(x, "x")
    N, C, H, W = x.shape
    y = torch.empty((N, C, H // k, W // k), dtype=x.dtype, device=x.device)
    mask = torch.empty(division_mask_bytes(x.numel()) // 4, dtype=torch.int32, device=x.device)
    rc = lib().division_maxpool_forward(x.data_ptr(), N, C, H, W, _dt(x.dtype), k, y.data_ptr(), mask.data_ptr(),
                                        mask.numel() * 4, _stream(stream))
    if rc:
        raise DivisionError(rc, "division_maxpool_forward")
    return y, mask


def division_maxpool_backward(mask: torch.Tensor, grad_out: torch.Tensor, shape, k: int, stream=None):
    """grad_in of shape `shape` (the pooled layer's input) from the location mask and grad_out."""
    _flat_ok(grad_out, "grad_out")
    N, C, H, W = shape
    if tuple(grad_out.shape) != (N, C, H // k, W // k):
        raise ValueError("grad_out has the wrong shape")
    out = torch.empty(tuple(shape), dtype=grad_out.dtype, device=grad_out.device)
    rc = lib().division_maxpool_backward(mask.data_ptr(), mask.numel() * mask.element_size(), grad_out.data_ptr(),
                                         N, C, H, W, _dt(grad_out.dtype), k, out.data_ptr(), _stream(stream))
    if rc:
        raise DivisionError(rc, "division_maxpool_backward")
    return out
