"""Seeded synthetic activation tensors shaped like the paper's CNN workloads.

This module only draws inputs.  It holds none of the codec's arithmetic and is
the one piece of code that the GPU path's tests, the CPU oracle's tests and the
benchmark all share: both sides are always fed the very same arrays.

The paper measures on ImageNet / CIFAR training runs (ResNet-50 at 224x224 with
batch 64, ResNet-18 on 32x32 CIFAR images; experiment-setting appendix).
Neither dataset nor trained weights are available here; these tensors take the
workloads' activation *shapes* and a post-ReLU value distribution and stand in
for the real activations.

Every config is a list of TensorSpec; `draw(spec, gen)` returns a float32
torch tensor on the host (bf16 specs are rounded to bfloat16 by the caller via
`.to(torch.bfloat16)`, round-to-nearest-even).  Draw order within a config is
the list order, from one torch.Generator seeded with the config's seed, so a
tensor's values depend on the ones drawn before it; `draw_config` does that.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterator, List, Tuple

import torch


@dataclass(frozen=True)
class TensorSpec:
    name: str
    shape: Tuple[int, int, int, int]   # N, C, H, W
    B: int                              # pooling block size
    b: int                              # HFC bit width
    dtype: str = "f32"                  # "f32" | "bf16"
    dist: str = "relu_normal"           # "relu_normal" | "relu_normal_gain" | "laplace_outliers"


def _rep(n, **kw):
    return [TensorSpec(name=f"{kw['name']}#{i}", **{k: v for k, v in kw.items() if k != "name"})
            for i in range(n)]


def config(idx: int) -> Tuple[int, List[TensorSpec]]:
    """Returns (generator seed, tensor specs) of workload `idx` (0..4)."""
    if idx == 0:    # one small tensor
        return 0, [TensorSpec("2x16x32x32", (2, 16, 32, 32), 8, 2)]
    if idx == 1:    # ResNet-18 / CIFAR shapes, batch 128
        n = 128
        return 1, (_rep(4, name="64x32x32", shape=(n, 64, 32, 32), B=4, b=2)
                   + _rep(4, name="128x16x16", shape=(n, 128, 16, 16), B=4, b=2)
                   + _rep(4, name="256x8x8", shape=(n, 256, 8, 8), B=4, b=2)
                   + _rep(4, name="512x4x4", shape=(n, 512, 4, 4), B=4, b=2))
    if idx == 2:    # ResNet-50 / ImageNet shapes, batch 64
        n = 64
        return 2, (_rep(1, name="64x112x112", shape=(n, 64, 112, 112), B=8, b=2)
                   + _rep(3, name="256x56x56", shape=(n, 256, 56, 56), B=8, b=2)
                   + _rep(4, name="512x28x28", shape=(n, 512, 28, 28), B=8, b=2)
                   + _rep(6, name="1024x14x14", shape=(n, 1024, 14, 14), B=8, b=2)
                   + _rep(3, name="2048x7x7", shape=(n, 2048, 7, 7), B=8, b=2))
    if idx == 3:    # one large bf16 tensor with per-channel gain
        return 3, [TensorSpec("256x256x56x56", (256, 256, 56, 56), 8, 2, "bf16", "relu_normal_gain")]
    if idx == 4:    # edge shapes, heavy tails, 4-bit codes
        n = 32
        return 4, [TensorSpec("512x7x7", (n, 512, 7, 7), 8, 4, "f32", "laplace_outliers"),
                   TensorSpec("1024x14x14", (n, 1024, 14, 14), 8, 4, "f32", "laplace_outliers"),
                   TensorSpec("96x55x55", (n, 96, 55, 55), 4, 4, "f32", "laplace_outliers")]
    raise ValueError("config index must be 0..4")


def draw(spec: TensorSpec, gen: torch.Generator, batch: int | None = None) -> torch.Tensor:
    """One float32 host tensor.  `batch` overrides N (reduced-size test cases)."""
    n, c, h, w = spec.shape
    if batch is not None:
        n = batch
    shape = (n, c, h, w)
    if spec.dist == "relu_normal":
        return torch.relu(torch.randn(shape, generator=gen, dtype=torch.float32))
    if spec.dist == "relu_normal_gain":
        gain = torch.empty(c, dtype=torch.float32).uniform_(0.1, 4.0, generator=gen)
        x = torch.relu(torch.randn(shape, generator=gen, dtype=torch.float32))
        return x * gain.view(1, c, 1, 1)
    if spec.dist == "laplace_outliers":
        u = torch.rand(shape, generator=gen, dtype=torch.float32) - 0.5
        x = -torch.sign(u) * torch.log1p(-2.0 * u.abs().clamp(max=0.49999997))
        mask = torch.rand(shape, generator=gen, dtype=torch.float32) < 0.001
        return torch.where(mask, x * 50.0, x)
    raise ValueError(spec.dist)


def draw_config(idx: int, batch: int | None = None) -> Iterator[Tuple[int, TensorSpec, torch.Tensor]]:
    """Yields (k, spec, float32 host tensor) in the config's draw order."""
    seed, specs = config(idx)
    gen = torch.Generator().manual_seed(seed)
    for k, spec in enumerate(specs):
        yield k, spec, draw(spec, gen, batch)


def codec_seed(config_idx: int, k: int) -> int:
    """The 64-bit codec seed used for tensor k of a config."""
    return (config_idx << 32) | k
