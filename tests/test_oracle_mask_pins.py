"""Pins of the oracle's 1-bit mask operators (Relu / Dropout, the paper's appendix on operator
compression) against things other than the oracle: numpy's own elementwise routines and bit
packing, the algebra of the listings, an independent big-integer evaluation of the random stream,
and binomial statistics."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from tests import pyref


def _bits(mask_words: np.ndarray, n: int) -> np.ndarray:
    return np.unpackbits(mask_words.view(np.uint8), bitorder="little")[:n].astype(bool)


def _values(rng, n):
    x = rng.standard_normal(n).astype(np.float32)
    x[::7] = 0.0
    x[3::11] = -0.0
    x[5::13] = np.float32(1e-45)          # smallest subnormal: positive, kept
    return x


@pytest.mark.parametrize("n", [0, 1, 31, 32, 33, 64, 1000, 4097])
def test_relu_forward_is_numpy_maximum_and_packbits(n):
    rng = np.random.default_rng(n)
    x = _values(rng, n)
    y, mask = oracle.relu_forward(x)
    assert mask.size == (n + 31) // 32
    keep = x > 0
    # Algorithm "Relu operator": V = sgn(H), out = V (.) H
    assert np.array_equal(y, np.where(keep, x, np.float32(0.0)))
    assert np.array_equal(y, np.maximum(x, np.float32(0.0)))                   # the textbook ReLU
    assert not np.signbit(y[~keep]).any()                                      # dropped values are +0
    ref = np.packbits(keep, bitorder="little")
    assert np.array_equal(mask.view(np.uint8)[:ref.size], ref)
    assert not mask.view(np.uint8)[ref.size:].any()                            # pad bits zero
    assert mask.size * 4 == oracle.mask_bytes(n)


def test_relu_nan_and_infinities():
    x = np.array([np.nan, np.inf, -np.inf, -1.0, 2.0], dtype=np.float32)
    y, mask = oracle.relu_forward(x)
    assert np.array_equal(_bits(mask, 5), [False, True, False, False, True])
    assert np.array_equal(y, np.array([0.0, np.inf, 0.0, 0.0, 2.0], dtype=np.float32))


def test_mask_backward_is_elementwise_product_with_the_indicator():
    rng = np.random.default_rng(7)
    n = 2500
    x = _values(rng, n)
    g = rng.standard_normal(n).astype(np.float32)
    _, mask = oracle.relu_forward(x)
    gin = oracle.mask_backward(mask, g)
    # Algorithm "Relu operator", backward: grad_in = V (.) grad_out
    assert np.array_equal(gin, np.where(x > 0, g, np.float32(0.0)))
    assert np.array_equal(gin, g * (x > 0).astype(np.float32) + np.float32(0.0))   # -0 * 0 folded to +0
    # all-ones and all-zero masks: identity and annihilation
    ones = np.full((n + 31) // 32, 0xFFFFFFFF, dtype=np.uint32)
    assert np.array_equal(oracle.mask_backward(ones, g), g)
    assert not oracle.mask_backward(np.zeros_like(ones), g).any()


def test_bf16_values_pass_through_bit_for_bit():
    rng = np.random.default_rng(9)
    xf = rng.standard_normal(777).astype(np.float32)
    xb = oracle.bf16_bits(xf)
    y, mask = oracle.relu_forward(xb, oracle.BF16)
    keep = oracle.bf16_to_f32(xb) > 0
    assert np.array_equal(y, np.where(keep, xb, np.uint16(0)))
    assert np.array_equal(_bits(mask, 777), keep)
    g = oracle.bf16_bits(rng.standard_normal(777).astype(np.float32))
    assert np.array_equal(oracle.mask_backward(mask, g, oracle.BF16), np.where(keep, g, np.uint16(0)))


def test_dropout_threshold_closed_form():
    for p, T in [(0.0, 0), (1.0, 65536), (0.5, 32768), (0.25, 16384), (1.0 / 65536, 1), (0.1, 6554),
                 (-0.3, 0), (2.0, 65536), (float("nan"), 0), (0.999999, 65536)]:
        assert oracle.dropout_threshold(p) == T, p
    for p in np.linspace(0, 1, 97):
        p32 = float(np.float32(p))
        assert oracle.dropout_threshold(p32) == int(Fraction(p32) * 65536 + Fraction(1, 2))   # exact rational floor
    # p * 65536 + 1/2 a hair below an integer: it must not be rounded up on the way (a binary32 sum would be)
    for eps in (2.0 ** -25, 2.0 ** -24):
        p32 = float(np.float32((0.5 - eps) / 65536))
        assert Fraction(p32) * 65536 + Fraction(1, 2) < 1
        assert oracle.dropout_threshold(p32) == 0, eps


@pytest.mark.parametrize("p", [0.0, 0.1, 0.5, 0.9, 1.0])
def test_dropout_mask_follows_the_independent_stream_evaluation(p):
    n, seed = 515, 0x1234_5678_9ABC_DEF0
    x = np.arange(1, n + 1, dtype=np.float32)
    y, mask = oracle.dropout_forward(x, p, seed)
    T = oracle.dropout_threshold(p)
    s = seed ^ 0xD509A5B3C2E1F047
    keep = np.array([pyref.rand16(s, 0, i) >= T for i in range(n)])
    assert np.array_equal(_bits(mask, n), keep)
    # Algorithm "Dropout operator": out = V (.) H, no rescaling
    assert np.array_equal(y, np.where(keep, x, np.float32(0.0)))
    if p == 0.0:
        assert keep.all()
    if p == 1.0:
        assert not keep.any()


def test_dropout_keep_rate_and_independence():
    n = 1 << 18
    x = np.ones(n, dtype=np.float32)
    for p in (0.1, 0.5, 0.8):
        _, m1 = oracle.dropout_forward(x, p, 11)
        _, m2 = oracle.dropout_forward(x, p, 12)
        k1, k2 = _bits(m1, n), _bits(m2, n)
        q = 1.0 - oracle.dropout_threshold(p) / 65536.0
        sd = (n * q * (1 - q)) ** 0.5
        assert abs(k1.sum() - n * q) < 5 * sd
        assert abs(k2.sum() - n * q) < 5 * sd
        # two seeds agree on about q^2 + (1-q)^2 of the positions, neighbours are uncorrelated
        agree = (k1 == k2).mean()
        assert abs(agree - (q * q + (1 - q) * (1 - q))) < 0.01
        c = np.corrcoef(k1[:-1], k1[1:])[0, 1]
        assert abs(c) < 0.01
        # same seed: same mask
        _, m3 = oracle.dropout_forward(x, p, 11)
        assert np.array_equal(m1, m3)


def test_dropout_stream_differs_from_the_codec_stream_of_the_same_seed():
    n, seed = 4096, 5
    x = np.ones(n, dtype=np.float32)
    _, m = oracle.dropout_forward(x, 0.5, seed)
    codec_bits = np.array([oracle.rand16(seed, 0, i) >= 32768 for i in range(n)])
    assert abs((_bits(m, n) == codec_bits).mean() - 0.5) < 0.05


# ---------------------------------------------------------------- Max-Pooling layer (kernel = stride = k)

import torch
import torch.nn.functional as F

MP_CASES = [((2, 3, 8, 8), 2), ((1, 2, 9, 7), 2), ((2, 2, 12, 9), 3), ((1, 1, 5, 5), 1), ((3, 1, 4, 6), 4),
            ((1, 2, 112, 112), 2), ((2, 1, 7, 7), 7), ((1, 1, 10, 13), 5)]


@pytest.mark.parametrize("shape,k", MP_CASES)
def test_maxpool_forward_is_the_library_pooling_with_its_argmax(shape, k):
    rng = np.random.default_rng(sum(shape) + k)
    x = rng.standard_normal(shape).astype(np.float32)         # no ties
    N, C, H, W = shape
    y, mask = oracle.maxpool_forward(x, k)
    ty, tidx = F.max_pool2d(torch.from_numpy(x), k, stride=k, return_indices=True)
    assert np.array_equal(y, ty.numpy())
    bits = _bits(mask, x.size).reshape(N * C, H * W)
    ref = np.zeros_like(bits)
    flat = tidx.numpy().reshape(N * C, -1)                      # indices inside each plane
    for p in range(N * C):
        ref[p, flat[p]] = True
    assert np.array_equal(bits, ref)
    # footnote of the algorithm: one location per window; rows / columns past the last window: none
    assert bits.sum() == N * C * (H // k) * (W // k)
    b4 = bits.reshape(N, C, H, W)
    assert not b4[:, :, (H // k) * k:, :].any() and not b4[:, :, :, (W // k) * k:].any()


@pytest.mark.parametrize("shape,k", MP_CASES)
def test_maxpool_backward_is_the_library_gradient(shape, k):
    rng = np.random.default_rng(17 * sum(shape) + k)
    x = rng.standard_normal(shape).astype(np.float32)
    N, C, H, W = shape
    g = rng.standard_normal((N, C, H // k, W // k)).astype(np.float32)
    _, mask = oracle.maxpool_forward(x, k)
    gin = oracle.maxpool_backward(mask, g, shape, k)
    tx = torch.from_numpy(x).requires_grad_(True)
    F.max_pool2d(tx, k, stride=k).backward(torch.from_numpy(g))
    assert np.array_equal(gin, tx.grad.numpy())
    # the listing's formula: V (.) (1_{k x k} (x) grad_out)
    up = np.repeat(np.repeat(g, k, 2), k, 3)
    full = np.zeros(shape, dtype=np.float32)
    full[:, :, :up.shape[2], :up.shape[3]] = up
    assert np.array_equal(gin, np.where(_bits(mask, x.size).reshape(shape), full, np.float32(0.0)))


def test_maxpool_ties_take_the_first_location_in_row_major_order():
    x = np.zeros((1, 1, 4, 4), dtype=np.float32)
    x[0, 0, 1, 1] = 5.0
    x[0, 0, 0, 3] = 2.0
    x[0, 0, 1, 2] = 2.0                      # ties with (0,3) in the top-right window; (0,3) comes first
    y, mask = oracle.maxpool_forward(x, 2)
    bits = _bits(mask, 16).reshape(4, 4)
    want = np.zeros((4, 4), dtype=bool)
    want[1, 1] = want[0, 3] = want[2, 0] = want[2, 2] = True       # all-zero windows mark their first element
    assert np.array_equal(bits, want)
    assert np.array_equal(y[0, 0], [[5.0, 2.0], [0.0, 0.0]])


def test_maxpool_bf16_passes_values_bit_for_bit():
    rng = np.random.default_rng(23)
    xf = rng.standard_normal((2, 3, 6, 10)).astype(np.float32)
    xb = oracle.bf16_bits(xf)
    y, mask = oracle.maxpool_forward(xb, 2, oracle.BF16)
    ty = F.max_pool2d(torch.from_numpy(oracle.bf16_to_f32(xb)), 2)
    assert np.array_equal(oracle.bf16_to_f32(y), ty.numpy())
