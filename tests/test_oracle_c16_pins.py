"""Pins of the oracle's paper-format mode (fp32 maps whose H^L, delta and Delta are cached as
bfloat16, Sec. 4.1): the paper's byte accounting, the bracketing invariants of the rounded
(delta, Delta), an exact-rational second formulation, the one-step error bound and unbiasedness."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from tests import pyref

C16 = oracle.F32_C16


def _rng(s):
    return np.random.default_rng(s)


def _maps(shape, seed, kind="relu"):
    x = _rng(seed).standard_normal(shape).astype(np.float32)
    if kind == "relu":
        x = np.maximum(x, 0)
    elif kind == "big":
        x = x * np.float32(1e6) + np.float32(3e7)
    elif kind == "tiny":
        x = x * np.float32(1e-20)
    return x


def test_byte_accounting_is_the_papers():
    # Sec. 4.1: (V^H, delta, h_max) cost N^2 Q/8 + 4 bytes per channel; H^L at B = 8 costs 0.8 % of H
    for N, Q in [(56, 2), (112, 2), (28, 4), (8, 8), (16, 2)]:
        lay = oracle.packed_layout(1, 1, N, N, 8, Q, C16)
        assert lay["codes_bytes"] + lay["meta_bytes"] == N * N * Q // 8 + 4
    lay = oracle.packed_layout(1, 1, 56, 56, 8, 2, C16)
    assert round(100 * lay["lfc_bytes"] / (4 * 56 * 56), 1) == 0.8
    assert round(100 * (56 * 56 * 2 / 8) / (4 * 56 * 56), 1) == 6.2          # V^H alone: Q/32
    # against the fp32-cached layout: 4 bytes less per plane and half the LFC
    a, b = oracle.packed_layout(3, 5, 28, 28, 8, 2, C16), oracle.packed_layout(3, 5, 28, 28, 8, 2, oracle.F32)
    assert a["codes_bytes"] == b["codes_bytes"] and 2 * a["meta_bytes"] == b["meta_bytes"] and 2 * a["lfc_bytes"] == b["lfc_bytes"]


@pytest.mark.parametrize("kind", ["relu", "plain", "big", "tiny"])
@pytest.mark.parametrize("b", [2, 4, 8])
def test_cached_delta_and_Delta_bracket_every_residual(kind, b):
    shape, B = (3, 4, 14, 14), 8
    x = _maps(shape, 7 + b, kind)
    p, d = oracle.compress(x, B, b, 3, C16, debug=True)
    s = oracle.split_packed(p, shape, B, b, C16)
    L = (1 << b) - 1
    assert s["meta"].dtype == np.uint16                                        # bfloat16 bit patterns
    delta = oracle.bf16_to_f32(s["meta"][:, 0]).astype(np.float64)
    Delta = oracle.bf16_to_f32(s["meta"][:, 1]).astype(np.float64)
    h = d["h"].reshape(12, -1).astype(np.float64)
    lo, hi = h.min(1), h.max(1)
    assert np.all(delta <= lo)                                                 # rounded down
    assert np.all(delta + L * Delta >= hi * (1 - 2.0 ** -23) - 2.0 ** -140)   # code range covers the maximum
    # and tight: within one bfloat16 step (2^-7 relative) of the unrounded values
    assert np.all(lo - delta <= np.abs(lo) * 2.0 ** -7 + 1e-300)
    rng = hi - delta
    assert np.all(Delta <= rng / L * (1 + 2.0 ** -7) + 1e-300)
    # pre-round values stay inside the code range, up to the few ulp the integer quantiser allows for
    t = d["t"].reshape(12, -1)
    assert t.min() >= 0 and t.max() <= L * (1 + 3 * 2.0 ** -24)
    # H^L is the block mean rounded to bfloat16
    up = np.repeat(np.repeat(oracle.bf16_to_f32(s["lfc"]).reshape(3, 4, 2, 2), B, 2), B, 3)[:, :, :14, :14]
    assert np.array_equal(d["h"], x - up)


@pytest.mark.parametrize("H,W,B,b", [(2, 2, 2, 2), (5, 7, 3, 4), (6, 6, 4, 4), (7, 7, 8, 2), (5, 6, 4, 8)])
def test_exact_rational_second_formulation(H, W, B, b):
    N, C = 2, 2
    x = _rng(300 + H * 31 + W * 7 + B).standard_normal((N, C, H, W)).astype(np.float32)
    seed = 0x0123456789ABCDEF
    p = oracle.compress(x, B, b, seed, C16)
    xh = oracle.decompress(p, x.shape, B, b, C16)
    s = oracle.split_packed(p, x.shape, B, b, C16)
    q = oracle.unpack_codes(s["codes"], H * W, b)
    for pl in range(N * C):
        xs = [Fraction(float(v)) for v in x.reshape(N * C, -1)[pl]]
        ref = pyref.codec_plane(xs, H, W, B, b, seed, pl, c16=True)
        assert [Fraction(float(v)) for v in oracle.bf16_to_f32(s["lfc"][pl]).ravel()] == ref["lfc"]
        assert Fraction(float(oracle.bf16_to_f32(s["meta"][pl, 0:1])[0])) == ref["delta"]
        assert Fraction(float(oracle.bf16_to_f32(s["meta"][pl, 1:2])[0])) == ref["Delta"]
        assert q[pl].tolist() == ref["codes"]
        assert [Fraction(float(v)) for v in xh.reshape(N * C, -1)[pl]] == ref["xhat"]


def test_decompress_is_dequant_plus_upsampled_lfc_with_the_cached_values():
    shape, B, b = (2, 3, 10, 14), 4, 4
    x = _maps(shape, 10, "plain")
    p = oracle.compress(x, B, b, 9, C16)
    xh = oracle.decompress(p, shape, B, b, C16)
    s = oracle.split_packed(p, shape, B, b, C16)
    q = oracle.unpack_codes(s["codes"], 140, b).reshape(shape).astype(np.float32)
    up = np.repeat(np.repeat(oracle.bf16_to_f32(s["lfc"]).reshape(2, 3, 3, 4), B, 2), B, 3)[:, :, :10, :14]
    m = oracle.bf16_to_f32(s["meta"])
    hh = q * m[:, 1].reshape(2, 3, 1, 1) + m[:, 0].reshape(2, 3, 1, 1)       # Sec. 4.2 with numpy fp32 ops
    assert np.array_equal(xh, up + hh)


@pytest.mark.parametrize("b", [2, 4, 8])
def test_one_step_error_bound_and_unbiasedness(b):
    shape, B = (2, 4, 16, 16), 8
    x = _maps(shape, 21, "relu")
    K = 300
    acc = np.zeros(shape, np.float64)
    for seed in range(K):
        p = oracle.compress(x, B, b, seed, C16)
        xh = oracle.decompress(p, shape, B, b, C16)
        acc += xh
        if seed == 0:
            s = oracle.split_packed(p, shape, B, b, C16)
            Delta = oracle.bf16_to_f32(s["meta"][:, 1]).reshape(2, 4, 1, 1).astype(np.float64)
            # stochastic rounding moves a value by less than one step (plus fp32 rounding of the sums)
            assert np.all(np.abs(xh - x.astype(np.float64)) <= Delta * (1 + 1e-5) + 1e-6)
    err = np.abs(acc / K - x.astype(np.float64))
    assert np.all(err <= 4.5 * Delta * 0.5 / K ** 0.5 + 1e-6)                 # E[xhat] = x


def test_degenerate_and_constant_planes():
    x = np.full((1, 2, 8, 8), 0.3, dtype=np.float32)
    x[0, 1] = 0.0
    p = oracle.compress(x, 8, 2, 1, C16)
    s = oracle.split_packed(p, x.shape, 8, 2, C16)
    xh = oracle.decompress(p, x.shape, 8, 2, C16)
    # all-zero plane: residual 0 = its own bfloat16 floor, range 0: Delta = 0, all codes 0, exact
    assert not s["codes"][1].any() and not s["meta"][1].any()
    assert np.array_equal(xh[0, 1], x[0, 1])
    # constant 0.3: the bfloat16 mean is off by up to 2^-9 relative, the constant residual is not a
    # bfloat16 value, so the plane is NOT degenerate; it comes back within one (tiny) step
    Delta = float(oracle.bf16_to_f32(s["meta"][0, 1:2])[0])
    assert 0 < Delta <= 0.3 * 2.0 ** -8
    assert np.all(np.abs(xh[0, 0] - x[0, 0]) <= Delta + 2.0 ** -24)      # one step plus the fp32 rounding of the sum
