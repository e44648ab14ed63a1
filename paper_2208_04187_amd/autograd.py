"""Algorithm 1 as a saved-tensor hook for torch.autograd.

Inside `with division_saved_tensors(B, b, seed):` every activation map that
autograd saves for the backward pass (N x C x H x W; also the N x C x L and
N x C x D x H x W maps of Appendix D) is replaced by its cached tuple (Algorithm
1, forward loop: AveragePooling, residual, Quant, Cache) and rebuilt when the
backward pass asks for it (backward loop: Dequant, UpSampling + add), so each
layer's gradients are estimated from the reconstructed map as in Sec. 4.2.
Parameters, small tensors and tensors that are not contiguous float32 /
bfloat16 device tensors of three to five dimensions are saved as they are.  Only calls the binding: all
arithmetic runs in the HIP library.
"""
from __future__ import annotations

import torch

from .binding import division_compress, division_compress_3d, division_decompress, division_decompress_3d


class _Cached:
    __slots__ = ("packed", "shape", "dtype", "B", "b", "c16")

    def __init__(self, packed, shape, dtype, B, b, c16):
        self.packed, self.shape, self.dtype, self.B, self.b, self.c16 = packed, shape, dtype, B, b, c16


class division_saved_tensors(torch.autograd.graph.saved_tensors_hooks):
    """Context manager.  `seed` selects the stochastic-rounding streams: the k-th map cached inside
    the context uses seed + k, so a training step is reproducible and no two maps share a stream.
    `c16` caches fp32 maps in the paper's format (bfloat16 H^L, delta, Delta); bfloat16 maps are
    cached in their own format either way."""

    def __init__(self, B: int = 8, b: int = 2, seed: int = 0, min_elements: int = 1024, c16: bool = False):
        self.cached_maps = 0        # maps cached so far
        self.cached_bytes = 0       # bytes of their packed buffers
        self.original_bytes = 0     # bytes the maps themselves would have held

        def pack(t: torch.Tensor):
            eligible = (t.is_cuda and t.dim() in (3, 4, 5) and t.dtype in (torch.float32, torch.bfloat16)
                        and t.is_contiguous() and t.numel() >= min_elements
                        and not isinstance(t, torch.nn.Parameter) and not (t.is_leaf and t.requires_grad))
            if not eligible:
                return t
            use16 = c16 and t.dtype == torch.float32
            src = t.detach()
            if src.dim() == 5:
                packed = division_compress_3d(src, B, b, seed + self.cached_maps, c16=use16)
            else:
                if src.dim() == 3:                       # Minibatch x Channel x N: the H = 1 case
                    src = src.unsqueeze(2)
                packed = division_compress(src, B, b, seed + self.cached_maps, c16=use16)
            self.cached_maps += 1
            self.cached_bytes += packed.numel()
            self.original_bytes += t.numel() * t.element_size()
            return _Cached(packed, tuple(t.shape), t.dtype, B, b, use16)

        def unpack(obj):
            if not isinstance(obj, _Cached):
                return obj
            if len(obj.shape) == 5:
                return division_decompress_3d(obj.packed, obj.shape, obj.B, obj.b, obj.dtype, c16=obj.c16)
            if len(obj.shape) == 3:
                n, c, length = obj.shape
                return division_decompress(obj.packed, (n, c, 1, length), obj.B, obj.b, obj.dtype, c16=obj.c16).view(obj.shape)
            return division_decompress(obj.packed, obj.shape, obj.B, obj.b, obj.dtype, c16=obj.c16)

        super().__init__(pack, unpack)
