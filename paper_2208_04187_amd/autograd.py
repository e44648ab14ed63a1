"""Algorithm 1 under torch.autograd: a saved-tensor hook that caches activation maps compressed, and the
operators whose backward pass needs an exact 1-bit mask instead of the map.

Inside `with division_saved_tensors(B, b, seed):` every activation map that autograd saves for the
backward pass (N x C x H x W; also the N x C x L and N x C x D x H x W maps of Appendix D) is replaced by
its cached tuple (Algorithm 1, forward loop: AveragePooling, residual, Quant, Cache) and rebuilt when the
backward pass asks for it (backward loop: Dequant, UpSampling + add), so each layer's gradients are
estimated from the reconstructed map as in Sec. 4.2.  Parameters, small tensors and tensors that are not
contiguous float32 / bfloat16 device tensors of three to five dimensions are saved as they are.

Launch pattern.  Algorithm 1 compresses once per layer; one library call per map is the slow way to issue
that (one short kernel per map, the machine filled and drained each time).  The hook therefore defers: a
map waits, uncompressed, until `group` maps (or `group_bytes` bytes) are waiting, and they go out in ONE
division_compress_maps call, which serves the maps that share a shape in one launch.  In the backward pass
the first map of such a group that is asked for rebuilds the whole group in one division_decompress_maps
call; the others are handed out when their turn comes.  `group=1` is the layer-by-layer pattern.

A map that several nodes save (the output of one layer is the input of the next) is compressed once.

Relu, Dropout and the Max-Pooling layer (appendix on operator compression) do not need the map in their
backward pass but a 1-bit mask, which is exact: DivisionReLU, DivisionDropout and DivisionMaxPool2d below
cache that mask and save no map of their own.  torch's own relu / max_pool2d save their output resp.
input; under the hook they would get the reconstructed map, whose signs and maxima differ from the true
ones.  Use the modules here for those operators.

Only calls the binding: all arithmetic runs in the HIP library.
"""
from __future__ import annotations

import weakref

import torch

from .binding import (division_compress_maps, division_decompress_maps, division_dropout_forward,
                      division_mask_backward, division_maxpool_backward, division_maxpool_forward,
                      division_packed_bytes, division_packed_bytes_3d, division_relu_forward)


class _Cached:
    """One cached map: waiting (src set), compressed (packed set), and for a while rebuilt (xhat set)."""
    __slots__ = ("src", "packed", "xhat", "shape", "dtype", "seed", "group", "saves", "__weakref__")

    def __init__(self, src, shape, dtype, seed):
        self.src, self.packed, self.xhat = src, None, None
        self.shape, self.dtype, self.seed = shape, dtype, seed
        self.group = None           # the entries that were compressed in the same call
        self.saves = 1              # how many nodes saved this map


def _as_map(t: torch.Tensor) -> torch.Tensor:
    """Minibatch x Channel x N maps are the H = 1 case of the 2-D calls."""
    return t.unsqueeze(2) if t.dim() == 3 else t


def _map_shape(shape):
    return (shape[0], shape[1], 1, shape[2]) if len(shape) == 3 else tuple(shape)


class division_saved_tensors(torch.autograd.graph.saved_tensors_hooks):
    """Context manager.  `seed` selects the stochastic-rounding streams: the k-th distinct map cached inside
    the context uses seed + k, so a training step is reproducible.  `c16` caches fp32 maps in the paper's
    format (bfloat16 H^L, delta, Delta); bfloat16 maps are cached in their own format either way.
    `group` / `group_bytes`: how many maps (bytes of maps) may wait uncompressed before they are compressed
    together; leaving the context compresses whatever still waits."""

    def __init__(self, B: int = 8, b: int = 2, seed: int = 0, min_elements: int = 1024, c16: bool = False,
                 group: int = 8, group_bytes: int = 1 << 31):
        self.B, self.b, self.c16 = B, b, c16
        self.cached_maps = 0        # distinct maps cached so far
        self.cached_bytes = 0       # bytes of their packed buffers
        self.original_bytes = 0     # bytes the maps themselves would have held
        self.compress_calls = 0     # library calls issued for them
        self.decompress_calls = 0
        self._pending = []
        self._pending_bytes = 0
        self._seen = {}             # (data_ptr, version, shape, dtype) -> (weak reference to the tensor, entry)
        group = max(1, int(group))

        def pack(t: torch.Tensor):
            eligible = (t.is_cuda and t.dim() in (3, 4, 5) and t.dtype in (torch.float32, torch.bfloat16)
                        and t.is_contiguous() and t.numel() >= min_elements
                        and not isinstance(t, torch.nn.Parameter) and not (t.is_leaf and t.requires_grad))
            if not eligible:
                return t
            key = (t.data_ptr(), t._version, tuple(t.shape), t.dtype)
            hit = self._seen.get(key)
            if hit is not None and (hit[1].src is not None or (hit[0] is not None and hit[0]() is not None)):
                # the memory cached under this key is still held (by the waiting entry or by the tensor
                # object that was saved), so this is the same map at the same version
                hit[1].saves += 1
                return hit[1]
            entry = _Cached(t.detach(), tuple(t.shape), t.dtype, seed + self.cached_maps)
            try:
                self._seen[key] = (weakref.ref(t), entry)
            except TypeError:
                self._seen[key] = (None, entry)
            use16 = c16 and t.dtype == torch.float32
            ms = _map_shape(entry.shape)
            nbytes = (division_packed_bytes_3d(*ms, B, b, t.dtype, use16) if len(ms) == 5
                      else division_packed_bytes(*ms, B, b, t.dtype, use16))
            self.cached_maps += 1
            self.cached_bytes += nbytes
            self.original_bytes += t.numel() * t.element_size()
            self._pending.append(entry)
            self._pending_bytes += t.numel() * t.element_size()
            if len(self._pending) >= group or self._pending_bytes >= group_bytes:
                self.flush()
            return entry

        def unpack(obj):
            if not isinstance(obj, _Cached):
                return obj
            if obj.src is not None:
                self.flush()                      # the backward pass has caught up with a waiting map
            if obj.xhat is None:
                # rebuild, in one call, every map of this one's group that is still to be handed out
                todo = [e for e in obj.group if e.xhat is None and e.saves > 0] if obj.group else []
                if obj not in todo:
                    todo.append(obj)
                outs = division_decompress_maps([e.packed for e in todo], [_map_shape(e.shape) for e in todo],
                                                B, b, [e.dtype for e in todo], c16=c16)
                self.decompress_calls += 1
                for e, y in zip(todo, outs):
                    e.xhat = y.view(e.shape)
            y = obj.xhat
            obj.saves -= 1
            if obj.saves <= 0:
                obj.xhat = None                   # handed out to every node that saved it
            return y

        super().__init__(pack, unpack)

    def flush(self):
        """Compresses the maps that wait, in one library call."""
        todo, self._pending, self._pending_bytes = self._pending, [], 0
        if not todo:
            return
        packed = division_compress_maps([_as_map(e.src) for e in todo], self.B, self.b, [e.seed for e in todo], c16=self.c16)
        self.compress_calls += 1
        for e, pk in zip(todo, packed):
            e.packed, e.src, e.group = pk, None, todo
        # keys of maps that no longer wait stay valid only while their tensor lives (checked on lookup)
        self._seen = {k: v for k, v in self._seen.items() if v[0] is not None and v[0]() is not None}

    def __enter__(self):
        super().__enter__()
        return self

    def __exit__(self, *args):
        self.flush()
        return super().__exit__(*args)


# ---------------------------------------------------------------- operators that cache a 1-bit mask

class _ReLU(torch.autograd.Function):
    """Relu operator of the appendix on operator compression: forward caches V = sgn(H) packed to one bit
    per element, backward is V (.) grad."""

    @staticmethod
    def forward(ctx, x):
        y, mask = division_relu_forward(x.contiguous())
        ctx.save_for_backward(mask)
        return y

    @staticmethod
    def backward(ctx, grad_out):
        (mask,) = ctx.saved_tensors
        return division_mask_backward(mask, grad_out.contiguous())


class _Dropout(torch.autograd.Function):
    """Dropout operator of the same appendix: V ~ Bernoulli(1 - p), no rescaling (as in the listing)."""

    @staticmethod
    def forward(ctx, x, p, seed):
        y, mask = division_dropout_forward(x.contiguous(), p, seed)
        ctx.save_for_backward(mask)
        return y

    @staticmethod
    def backward(ctx, grad_out):
        (mask,) = ctx.saved_tensors
        return division_mask_backward(mask, grad_out.contiguous()), None, None


class _MaxPool2d(torch.autograd.Function):
    """Max-Pooling layer of the same appendix, kernel size = stride = k: V marks each window's maximum."""

    @staticmethod
    def forward(ctx, x, k):
        y, mask = division_maxpool_forward(x.contiguous(), k)
        ctx.save_for_backward(mask)
        ctx.in_shape, ctx.k = tuple(x.shape), k
        return y

    @staticmethod
    def backward(ctx, grad_out):
        (mask,) = ctx.saved_tensors
        return division_maxpool_backward(mask, grad_out.contiguous(), ctx.in_shape, ctx.k), None


class DivisionReLU(torch.nn.Module):
    def forward(self, x):
        return _ReLU.apply(x)


class DivisionMaxPool2d(torch.nn.Module):
    def __init__(self, kernel_size: int):
        super().__init__()
        self.k = int(kernel_size)

    def forward(self, x):
        return _MaxPool2d.apply(x, self.k)


class DivisionDropout(torch.nn.Module):
    """Keeps an element with probability 1 - p while training; the mask of call number n of this module
    comes from seed + n.  Identity in eval mode."""

    def __init__(self, p: float = 0.5, seed: int = 0):
        super().__init__()
        self.p, self.seed, self.calls = float(p), int(seed), 0

    def forward(self, x):
        if not self.training or self.p == 0.0:
            return x
        self.calls += 1
        return _Dropout.apply(x, self.p, self.seed + self.calls)
