"""Pins of the oracle's 3-D maps (Appendix D: AveragePooling3D / UpSampling3D, the same Quant).

The 3-D code path is checked against things other than itself: the library's 3-D pooling and
nearest up-sampling, an exact-rational re-derivation that finds blocks by coordinate search,
the 2-D oracle (pinned on its own) on volumes with one degenerate dimension, and symmetries of
cubic blocks.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from tests import pyref


def _rng(seed):
    return np.random.default_rng(seed)


VOLUMES = [((2, 3, 8, 8, 8), 4), ((1, 2, 5, 9, 13), 4), ((2, 2, 6, 10, 7), 3), ((1, 3, 16, 12, 20), 8),
           ((1, 2, 3, 20, 20), 8), ((2, 1, 9, 4, 6), 8), ((1, 1, 17, 5, 3), 2)]


@pytest.mark.parametrize("shape,B", VOLUMES)
def test_lfc_is_the_librarys_3d_average_pooling_and_residual_its_upsampling(shape, B):
    N, C, D, H, W = shape
    x = _rng(sum(shape) + B).standard_normal(shape).astype(np.float32)
    p, dbg = oracle.compress(x, B, 2, 17, debug=True)
    lfc = oracle.split_packed(p, shape, B, 2)["lfc"].reshape(N, C, -(-D // B), -(-H // B), -(-W // B))
    k = (min(B, D), min(B, H), min(B, W))          # a dimension shorter than B is one window
    ref = F.avg_pool3d(torch.from_numpy(x).double(), k, stride=k, ceil_mode=True, count_include_pad=False).float().numpy()
    assert lfc.shape == ref.shape
    assert np.array_equal(lfc, ref)
    up = torch.from_numpy(lfc).repeat_interleave(B, 2).repeat_interleave(B, 3).repeat_interleave(B, 4)[:, :, :D, :H, :W]
    if D % B == 0 and H % B == 0 and W % B == 0:
        # the paper's floor(N/B)^3 shape and the library's nearest interpolation
        assert lfc.shape[2:] == (D // B, H // B, W // B)
        assert torch.equal(up, F.interpolate(torch.from_numpy(lfc), size=(D, H, W), mode="nearest"))
    assert np.array_equal(dbg["h"], x - up.numpy())
    # Sec. 4.2 with numpy fp32 operations
    s = oracle.split_packed(p, shape, B, 2)
    q = oracle.unpack_codes(s["codes"], D * H * W, 2).reshape(shape).astype(np.float32)
    hh = q * s["meta"][:, 1].reshape(N, C, 1, 1, 1) + s["meta"][:, 0].reshape(N, C, 1, 1, 1)
    assert np.array_equal(oracle.decompress(p, shape, B, 2), up.numpy() + hh)


@pytest.mark.parametrize("dims,B,b", [((2, 2, 2), 2, 2), ((3, 4, 5), 2, 2), ((4, 3, 5), 3, 4), ((5, 4, 3), 4, 8),
                                      ((2, 5, 7), 8, 2), ((6, 2, 4), 1, 4)])
def test_brute_force_exact_rational_volume(dims, B, b):
    N, C = 2, 2
    x = _rng(300 + sum(dims) * 7 + B).standard_normal((N, C) + dims).astype(np.float32)
    x[0, 1] = np.round(x[0, 1] * 4) / 4
    seed = 0x0123456789ABCDEF
    p = oracle.compress(x, B, b, seed)
    xh = oracle.decompress(p, x.shape, B, b)
    s = oracle.split_packed(p, x.shape, B, b)
    n = int(np.prod(dims))
    q = oracle.unpack_codes(s["codes"], n, b)
    for pl in range(N * C):
        xs = [Fraction(float(v)) for v in x.reshape(N * C, -1)[pl]]
        ref = pyref.codec_volume(xs, dims, B, b, seed, pl)
        assert [Fraction(float(v)) for v in s["lfc"][pl].ravel()] == ref["lfc"]
        assert Fraction(float(s["meta"][pl, 0])) == ref["delta"]
        assert Fraction(float(s["meta"][pl, 1])) == ref["Delta"]
        assert q[pl].tolist() == ref["codes"]
        assert [Fraction(float(v)) for v in xh.reshape(N * C, -1)[pl]] == ref["xhat"]


def test_exact_rational_volume_agrees_with_the_plane_version_on_2d():
    # the two test-side formulations are themselves consistent where both apply
    x = _rng(5).standard_normal(35).astype(np.float32)
    xs = [Fraction(float(v)) for v in x]
    a = pyref.codec_plane(xs, 5, 7, 3, 4, 99, 2)
    b = pyref.codec_volume(xs, (5, 7), 3, 4, 99, 2)
    assert a["lfc"] == b["lfc"] and a["codes"] == b["codes"] and a["xhat"] == b["xhat"]


@pytest.mark.parametrize("dt", [oracle.F32, oracle.BF16, oracle.F32_C16])
@pytest.mark.parametrize("A,Bd,B,b", [(9, 14, 4, 2), (20, 6, 8, 4), (7, 7, 8, 2), (12, 30, 12, 8)])
def test_volume_with_one_degenerate_dimension_is_the_2d_codec(A, Bd, B, b, dt):
    # every element keeps its flat index, so the packed buffers are equal byte for byte
    xf = _rng(A * 100 + Bd).standard_normal((2, 3, A, Bd)).astype(np.float32)
    x = oracle.bf16_bits(xf) if dt == oracle.BF16 else xf
    ref = oracle.compress(x, B, b, 31, dt)
    for shape5 in [(2, 3, 1, A, Bd), (2, 3, A, 1, Bd), (2, 3, A, Bd, 1)]:
        p = oracle.compress(x.reshape(shape5), B, b, 31, dt)
        assert np.array_equal(p, ref), shape5
        assert np.array_equal(oracle.decompress(p, shape5, B, b, dt).reshape(x.shape), oracle.decompress(ref, x.shape, B, b, dt))


@pytest.mark.parametrize("perm", [(0, 1, 2, 4, 3), (0, 1, 3, 2, 4), (0, 1, 4, 3, 2), (0, 1, 3, 4, 2)])
def test_cubic_blocks_commute_with_permutations_of_the_map_axes(perm):
    shape, B = (2, 2, 6, 10, 7), 4
    x = _rng(77).standard_normal(shape).astype(np.float32) * 3
    xt = np.ascontiguousarray(x.transpose(perm))
    a = oracle.split_packed(oracle.compress(x, B, 4, 1), shape, B, 4)
    bt = oracle.split_packed(oracle.compress(xt, B, 4, 1), xt.shape, B, 4)
    lfc_a = a["lfc"].reshape(2, 2, 2, 3, 2)
    assert np.array_equal(np.ascontiguousarray(lfc_a.transpose(perm)).reshape(bt["lfc"].shape), bt["lfc"])
    assert np.array_equal(a["meta"], bt["meta"])          # min / max of the residual do not depend on the order


def test_block_constant_volume_has_zero_residual_and_B1_is_identity():
    B = 4
    small = _rng(3).standard_normal((2, 3, 2, 3, 2)).astype(np.float32)
    x = np.ascontiguousarray(np.repeat(np.repeat(np.repeat(small, B, 2), B, 3), B, 4)[:, :, :7, :10, :8])
    p, dbg = oracle.compress(x, B, 2, 5, debug=True)
    s = oracle.split_packed(p, x.shape, B, 2)
    assert not dbg["h"].any() and not s["codes"].any() and not s["meta"].any()
    assert np.array_equal(s["lfc"], small.reshape(6, 2, 3, 2))
    assert np.array_equal(oracle.decompress(p, x.shape, B, 2), x)
    y = _rng(4).standard_normal((1, 2, 3, 5, 4)).astype(np.float32)
    p1 = oracle.compress(y, 1, 4, 5)
    assert np.array_equal(oracle.decompress(p1, y.shape, 1, 4), y)
    assert np.array_equal(oracle.split_packed(p1, y.shape, 1, 4)["lfc"].reshape(y.shape), y)


@pytest.mark.parametrize("b", [2, 4, 8])
def test_volume_error_within_one_step_and_layout_closed_form(b):
    shape, B = (2, 3, 9, 11, 6), 4
    N, C, D, H, W = shape
    x = _rng(b).standard_normal(shape).astype(np.float32)
    p = oracle.compress(x, B, b, 8)
    s = oracle.split_packed(p, shape, B, b)
    xh = oracle.decompress(p, shape, B, b)
    Delta = s["meta"][:, 1].reshape(N, C, 1, 1, 1).astype(np.float64)
    assert np.all(np.abs(xh.astype(np.float64) - x) <= Delta * (1 + 1e-6) + 1e-6)
    lay = oracle.packed_layout_3d(N, C, D, H, W, B, b)
    n = D * H * W
    assert lay["codes_bytes"] == 4 * N * C * -(-n * b // 32)             # N^3 Q / 8 bytes per channel, in whole words
    assert lay["meta_bytes"] == 8 * N * C
    assert lay["lfc_bytes"] == 4 * N * C * 3 * 3 * 2
    assert lay["meta_off"] == -(-lay["codes_bytes"] // 16) * 16
    assert oracle.packed_bytes_3d(N, C, D, H, W, B, b) == len(p)
    assert oracle.packed_bytes_3d(N, C, 0, H, W, B, b) == 0
