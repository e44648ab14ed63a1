"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests needs a GPU.  They check the oracle against: a worked
example derived by hand from Eq. (quantization) and the reconstruction
equation; the invariants the method implies; PyTorch's pooling / upsampling
as the textbook special case; an exact-rational brute force on tiny inputs;
the byte accounting the paper prints; and statistical properties of the
random source.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from tests import pyref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _roundtrip(x, B, b, seed, dt=oracle.F32):
    p = oracle.compress(x, B, b, seed, dt)
    return p, oracle.decompress(p, x.shape, B, b, dt)


# ---------------------------------------------------------------- T1 worked examples

def test_worked_example_2x2_b2():
    # Eq. (quantization) by hand: lfc = 1.5, h = [-1.5,-.5,.5,1.5], delta = -1.5,
    # range 3, Delta = 1, t = [0,1,2,3]: integers are fixed points of the
    # stochastic rounding, so the codes are [0,1,2,3] for every seed.
    x = np.array([[[[0, 1], [2, 3]]]], np.float32)
    for seed in (0, 1, 2, 12345, 2 ** 63 + 5):
        p, xh = _roundtrip(x, 2, 2, seed)
        s = oracle.split_packed(p, x.shape, 2, 2)
        assert s["codes"].tolist() == [[0xE4]]
        assert s["meta"].tolist() == [[-1.5, 1.0]]
        assert s["lfc"].tolist() == [[[1.5]]]
        assert np.array_equal(xh, x)


def test_worked_example_1bit_codes():
    # Q = 1: L = 1, the two codes are the plane's extremes.  A 2 x 4 plane that is one block holding
    # {0, 4} only: mean 2, h = -+2, delta = -2, range 4, Delta = 4, t in {0, 1}: fixed points of the
    # rounding, so code = (x == 4) for every seed, 8 codes in the low byte of one word, and xhat = x.
    x = np.array([[[[0, 4, 4, 0], [4, 0, 0, 4]]]], np.float32)
    for seed in (0, 3, 2 ** 40 + 1):
        p, xh = _roundtrip(x, 4, 1, seed)
        s = oracle.split_packed(p, x.shape, 4, 1)
        assert s["codes"].tolist() == [[0b10010110]]
        assert s["meta"].tolist() == [[-2.0, 4.0]]
        assert s["lfc"].tolist() == [[[2.0]]]
        assert np.array_equal(xh, x)
    # a value a quarter of the way up is coded 1 with probability 1/4 (u uniform on 65536 steps)
    y = np.array([[[[0, 4, 1, 3]]]], np.float32)              # mean 2, h = [-2, 2, -1, 1], t = [0, 1, 1/4, 3/4]
    ones = np.zeros(4)
    n = 4000
    for seed in range(n):
        q = oracle.unpack_codes(oracle.split_packed(oracle.compress(y, 4, 1, seed), y.shape, 4, 1)["codes"], 4, 1)[0]
        ones += q
    assert ones[0] == 0 and ones[1] == n
    assert abs(ones[2] / n - 0.25) < 0.03 and abs(ones[3] / n - 0.75) < 0.03


def test_worked_example_4x4_b4():
    # one 4x4 block holding the ramp 0..15: mean 7.5, range 15, Delta 1, codes 0..15
    x = np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4)
    for seed in (0, 7, 99):
        p, xh = _roundtrip(x, 4, 4, seed)
        s = oracle.split_packed(p, x.shape, 4, 4)
        assert s["codes"].tolist() == [[0x76543210, 0xFEDCBA98]]
        assert s["meta"].tolist() == [[-7.5, 1.0]]
        assert np.array_equal(xh, x)


def test_worked_example_two_blocks_distinct_means():
    # 1x4 map, B=2: blocks {0,2} and {10,16}; lfc = [1,13]; h = [-1,1,-3,3];
    # delta=-3, range 6, Delta=2 (b=2), t = [1,2,0,3] -> codes fixed for any seed.
    x = np.array([[[[0, 2, 10, 16]]]], np.float32)
    p, xh = _roundtrip(x, 2, 2, 5)
    s = oracle.split_packed(p, x.shape, 2, 2)
    assert s["lfc"].ravel().tolist() == [1.0, 13.0]
    assert s["meta"].tolist() == [[-3.0, 2.0]]
    assert s["codes"].tolist() == [[1 | 2 << 2 | 0 << 4 | 3 << 6]]
    assert np.array_equal(xh, x)


# ---------------------------------------------------------------- I1..I6 invariants

@pytest.mark.parametrize("b", [2, 4, 8])
def test_B1_lfc_is_x_and_roundtrip_exact(b):
    x = _rng(1).standard_normal((2, 3, 5, 7)).astype(np.float32)
    p, xh = _roundtrip(x, 1, b, 3)
    s = oracle.split_packed(p, x.shape, 1, b)
    assert np.array_equal(s["lfc"].reshape(x.shape).view(np.uint32), x.view(np.uint32))
    assert not s["codes"].any()
    assert np.all(s["meta"] == 0.0)
    assert np.array_equal(xh.view(np.uint32), x.view(np.uint32))


@pytest.mark.parametrize("shape,B", [((2, 2, 8, 8), 4), ((1, 3, 7, 10), 4), ((2, 1, 14, 14), 8), ((1, 2, 5, 5), 8)])
def test_block_constant_gives_zero_hfc(shape, B):
    N, C, H, W = shape
    LH, LW = -(-H // B), -(-W // B)
    vals = _rng(2).standard_normal((N, C, LH, LW)).astype(np.float32)
    x = np.repeat(np.repeat(vals, B, 2), B, 3)[:, :, :H, :W].copy()
    p, d = oracle.compress(x, B, 2, 11, debug=True)
    s = oracle.split_packed(p, shape, B, 2)
    assert np.array_equal(s["lfc"].reshape(N, C, LH, LW), vals)     # mean of a constant block is the constant
    assert not d["h"].any()                                          # HFC identically zero
    assert not s["codes"].any() and np.all(s["meta"][:, 1] == 0)
    assert np.array_equal(oracle.decompress(p, shape, B, 2), x)


@pytest.mark.parametrize("b", [1, 2, 4, 8])
@pytest.mark.parametrize("shape,B", [((2, 4, 16, 16), 8), ((1, 5, 7, 7), 8), ((2, 3, 14, 14), 8), ((1, 2, 55, 55), 4)])
def test_reconstruction_error_bounded_by_one_step(shape, B, b):
    x = np.maximum(_rng(3).standard_normal(shape), 0).astype(np.float32)
    p, xh = _roundtrip(x, B, b, 17)
    Delta = oracle.split_packed(p, shape, B, b)["meta"][:, 1].reshape(shape[0], shape[1], 1, 1)
    err = np.abs(xh.astype(np.float64) - x)
    bound = Delta.astype(np.float64) * (1 + 1e-5) + 4 * np.spacing(np.abs(x) + 1)
    assert np.all(err <= bound)
    # and the error is not trivially zero: stochastic rounding moves most elements
    assert (err > 0).mean() > 0.3


def test_min_gets_code0_max_gets_top_code_for_every_seed():
    rng = _rng(4)
    for b in (2, 4, 8):
        L = (1 << b) - 1
        x = rng.standard_normal((4, 6, 9, 9)).astype(np.float32) * rng.uniform(1e-3, 1e3, (4, 6, 1, 1)).astype(np.float32)
        for seed in range(40):
            p, d = oracle.compress(x, 4, b, seed, debug=True)
            q = oracle.unpack_codes(oracle.split_packed(p, x.shape, 4, b)["codes"], 81, b)
            h = d["h"].reshape(24, 81)
            assert np.all(q[np.arange(24), h.argmin(1)] == 0)
            assert np.all(q[np.arange(24), h.argmax(1)] == L)


def test_scale_top_is_exact_for_many_ranges():
    # the one-ulp bump of the scale guarantees fl(range*inv) >= L: max -> code L.
    rng = _rng(5)
    for b in (2, 4, 8):
        L = (1 << b) - 1
        for _ in range(300):
            hi = np.float32(rng.uniform(0.5, 2.0) * 2.0 ** rng.integers(-20, 20))
            x = np.array([[[[0, hi, hi / 3, hi / 7]]]], np.float32)
            p, d = oracle.compress(x, 1000, b, 1, debug=True)
            hmax = d["h"].argmax()
            assert d["t"].ravel()[hmax] >= L
            q = oracle.unpack_codes(oracle.split_packed(p, x.shape, 1000, b)["codes"], 4, b)
            assert q[0, hmax] == L and q[0, d["h"].argmin()] == 0


def test_unbiased_over_seeds():
    # E[dequantised HFC] = HFC with the positions fixed and the seed varying
    # (second footnote of Eq. (quantization)).
    K, b, B = 4096, 2, 4
    x = np.maximum(_rng(6).standard_normal((1, 2, 8, 8)), 0).astype(np.float32)
    _, d0 = oracle.compress(x, B, b, 0, debug=True)
    h, t = d0["h"].astype(np.float64), d0["t"].astype(np.float64)
    acc = np.zeros(x.shape, np.float64)
    for seed in range(K):
        p = oracle.compress(x, B, b, seed)
        s = oracle.split_packed(p, x.shape, B, b)
        q = oracle.unpack_codes(s["codes"], 64, b).reshape(x.shape).astype(np.float64)
        acc += q * s["meta"][:, 1].reshape(1, 2, 1, 1).astype(np.float64) + s["meta"][:, 0].reshape(1, 2, 1, 1)
    mean = acc / K
    Delta = s["meta"][:, 1].reshape(1, 2, 1, 1).astype(np.float64)
    f = t - np.floor(t)
    sigma = Delta * np.sqrt(f * (1 - f) / K)
    assert np.all(np.abs(mean - h) <= 4.5 * sigma + Delta * 2.0 ** -16 + 1e-6)
    z = (mean - h)[sigma > 0] / sigma[sigma > 0]
    assert abs(z.mean()) < 4 / math.sqrt(z.size) and 0.7 < z.std() < 1.3
    # the footnote's literal wording (round DOWN w.p. frac) would be biased:
    # its mean would sit at floor+ (1-f), i.e. off by (1-2f)*Delta
    wrong = (np.floor(t) + (1 - f)) * Delta + s["meta"][:, 0].reshape(1, 2, 1, 1)
    assert np.abs(wrong - h).max() > 0.3 * Delta.min()


def test_round_up_probability_is_frac():
    # a plane [0, f*3, 3] with B huge: lfc = mean; t of the middle element is
    # known; over seeds it must round up with probability frac(t).
    x = np.array([[[[0.0, 1.3, 3.0, 0.2]]]], np.float32)
    ups, n = np.zeros(4), 3000
    _, d = oracle.compress(x, 99, 2, 0, debug=True)
    t = d["t"].ravel().astype(np.float64)
    for seed in range(n):
        p = oracle.compress(x, 99, 2, seed)
        q = oracle.unpack_codes(oracle.split_packed(p, x.shape, 99, 2)["codes"], 4, 2)[0]
        ups += q > np.floor(t)
    f = t - np.floor(t)
    assert np.all(np.abs(ups / n - f) < 4 * np.sqrt(f * (1 - f) / n) + 1e-3)


def test_deterministic_and_seed_sensitive():
    x = np.maximum(_rng(7).standard_normal((2, 3, 12, 12)), 0).astype(np.float32)
    a = oracle.compress(x, 4, 2, 42)
    assert np.array_equal(a, oracle.compress(x, 4, 2, 42))
    assert np.array_equal(a, oracle.compress(x, 4, 2, 42, threads=4))
    bb = oracle.compress(x, 4, 2, 43)
    sa, sb = oracle.split_packed(a, x.shape, 4, 2), oracle.split_packed(bb, x.shape, 4, 2)
    assert np.array_equal(sa["lfc"], sb["lfc"]) and np.array_equal(sa["meta"], sb["meta"])
    assert not np.array_equal(sa["codes"], sb["codes"])
    # high seed word matters too
    cc = oracle.compress(x, 4, 2, 42 + (1 << 32))
    assert not np.array_equal(sa["codes"], oracle.split_packed(cc, x.shape, 4, 2)["codes"])


# ---------------------------------------------------------------- X1 library special cases

@pytest.mark.parametrize("shape,B", [((2, 3, 16, 16), 8), ((2, 3, 16, 16), 4), ((1, 4, 14, 14), 8),
                                     ((1, 4, 7, 7), 8), ((2, 2, 55, 55), 4), ((1, 2, 9, 13), 3), ((1, 1, 28, 28), 8)])
def test_lfc_matches_library_avg_pool_and_upsampling(shape, B):
    N, C, H, W = shape
    x = _rng(8).standard_normal(shape).astype(np.float32)
    p, d = oracle.compress(x, B, 2, 0, debug=True)
    lfc = oracle.split_packed(p, shape, B, 2)["lfc"].reshape(N, C, -(-H // B), -(-W // B))
    kh, kw = min(B, H), min(B, W)           # footnote of Sec. 4.1: map smaller than B -> window = map
    ref = F.avg_pool2d(torch.from_numpy(x).double(), (kh, kw), stride=(kh, kw), ceil_mode=True,
                       count_include_pad=False).float().numpy()
    assert lfc.shape == ref.shape
    assert np.array_equal(lfc, ref)
    up = torch.from_numpy(lfc).repeat_interleave(B, 2).repeat_interleave(B, 3)[:, :, :H, :W]
    if H % B == 0 and W % B == 0:
        assert torch.equal(up, F.interpolate(torch.from_numpy(lfc), size=(H, W), mode="nearest"))
    assert np.array_equal(d["h"], x - up.numpy())


@pytest.mark.parametrize("L,B", [(64, 8), (197, 8), (128, 16), (50, 64), (96, 12)])
def test_1d_maps_are_the_H_equal_1_case(L, B):
    # Appendix D, AveragePooling1D / UpSampling1D: a Minibatch x Channel x N map is the 2-D codec on
    # Minibatch x Channel x 1 x N; checked against the library's 1-D pooling and nearest up-sampling
    N, C = 3, 5
    x = _rng(40 + L).standard_normal((N, C, 1, L)).astype(np.float32)
    p, d = oracle.compress(x, B, 2, 3, debug=True)
    lfc = oracle.split_packed(p, x.shape, B, 2)["lfc"].reshape(N, C, -(-L // B))
    k = min(B, L)
    ref = F.avg_pool1d(torch.from_numpy(x[:, :, 0, :]).double(), k, stride=k, ceil_mode=True,
                       count_include_pad=False).float().numpy()
    assert np.array_equal(lfc, ref)
    if L % B == 0:
        # the paper's floor(N/B) shape and the library's nearest interpolation
        assert lfc.shape[-1] == L // B
        up = F.interpolate(torch.from_numpy(lfc), size=L, mode="nearest").numpy()
        assert np.array_equal(d["h"][:, :, 0, :], x[:, :, 0, :] - up)


def test_map_smaller_than_block_is_one_window():
    # Sec. 4.1 footnote: N < B gives a 1x1 LFC equal to the plane mean
    x = _rng(9).standard_normal((3, 4, 7, 7)).astype(np.float32)
    p = oracle.compress(x, 8, 2, 0)
    lfc = oracle.split_packed(p, x.shape, 8, 2)["lfc"]
    assert lfc.shape == (12, 1, 1)
    assert np.array_equal(lfc.ravel(), x.astype(np.float64).mean((2, 3)).astype(np.float32).ravel())


def test_decompress_is_dequant_plus_upsampled_lfc():
    # Sec. 4.2: Delta*V+delta, then + UpSampling(H^L), evaluated with numpy fp32 ops
    shape, B, b = (2, 3, 10, 14), 4, 4
    x = _rng(10).standard_normal(shape).astype(np.float32)
    p, xh = _roundtrip(x, B, b, 9)
    s = oracle.split_packed(p, shape, B, b)
    q = oracle.unpack_codes(s["codes"], 140, b).reshape(shape).astype(np.float32)
    up = np.repeat(np.repeat(s["lfc"].reshape(2, 3, 3, 4), B, 2), B, 3)[:, :, :10, :14]
    hh = q * s["meta"][:, 1].reshape(2, 3, 1, 1) + s["meta"][:, 0].reshape(2, 3, 1, 1)
    assert np.array_equal(xh, up + hh)


# ---------------------------------------------------------------- X2 exact-rational brute force

@pytest.mark.parametrize("H,W,B,b", [(2, 2, 2, 2), (3, 5, 2, 2), (5, 7, 3, 4), (4, 4, 1, 2), (5, 7, 8, 2), (5, 7, 3, 1), (6, 11, 4, 1),
                                     (6, 6, 4, 4), (7, 7, 8, 4), (3, 9, 4, 2), (5, 6, 4, 8), (7, 7, 8, 8)])
def test_brute_force_exact_rational(H, W, B, b):
    rng = _rng(100 + H * 31 + W * 7 + B)
    N, C = 2, 2
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    x[0, 0] = np.round(x[0, 0] * 8) / 8                       # an exactly-summable plane too
    seed = 0xABCDEF0123456789
    p = oracle.compress(x, B, b, seed)
    xh = oracle.decompress(p, x.shape, B, b)
    s = oracle.split_packed(p, x.shape, B, b)
    q = oracle.unpack_codes(s["codes"], H * W, b)
    for pl in range(N * C):
        xs = [Fraction(float(v)) for v in x.reshape(N * C, -1)[pl]]
        ref = pyref.codec_plane(xs, H, W, B, b, seed, pl)
        assert [Fraction(float(v)) for v in s["lfc"][pl].ravel()] == ref["lfc"]
        assert Fraction(float(s["meta"][pl, 0])) == ref["delta"]
        assert Fraction(float(s["meta"][pl, 1])) == ref["Delta"]
        assert q[pl].tolist() == ref["codes"]
        assert [Fraction(float(v)) for v in xh.reshape(N * C, -1)[pl]] == ref["xhat"]


def test_brute_force_bf16_residual_against_stored_lfc():
    # bf16 input: LFC is rounded to bf16 and the residual is taken against the
    # rounded value, so the one-step error bound still holds after bf16 output rounding.
    rng = _rng(11)
    xf = np.maximum(rng.standard_normal((2, 3, 8, 8)), 0).astype(np.float32)
    xb = oracle.bf16_bits(xf)
    p, d = oracle.compress(xb, 4, 2, 5, dt=oracle.BF16, debug=True)
    s = oracle.split_packed(p, xb.shape, 4, 2, dt=oracle.BF16)
    lfc = oracle.bf16_to_f32(s["lfc"]).reshape(2, 3, 2, 2)
    exact = oracle.bf16_to_f32(xb).astype(np.float64).reshape(2, 3, 2, 4, 2, 4).mean((3, 5))
    assert np.array_equal(s["lfc"].reshape(2, 3, 2, 2), oracle.bf16_bits(exact.astype(np.float32)))
    up = np.repeat(np.repeat(lfc, 4, 2), 4, 3)
    assert np.array_equal(d["h"], oracle.bf16_to_f32(xb) - up)
    xh = oracle.bf16_to_f32(oracle.decompress(p, xb.shape, 4, 2, dt=oracle.BF16))
    Delta = s["meta"][:, 1].reshape(2, 3, 1, 1).astype(np.float64)
    x64 = oracle.bf16_to_f32(xb).astype(np.float64)
    assert np.all(np.abs(xh - x64) <= Delta * (1 + 1e-5) + np.abs(x64) * 2.0 ** -8 + 1e-6)


# ---------------------------------------------------------------- Y1 byte accounting

def _paper_values():
    vals = {}
    with open(os.path.join(GOLDEN, "paper_values.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if "=" in line:
                k, v = line.split("=", 1)
                vals[k.strip()] = v.strip()
    return vals


def test_layout_closed_form_and_config_sizes():
    def closed(N, C, H, W, B, b, es):
        a16 = lambda v: (v + 15) // 16 * 16
        P, WPP = N * C, -(-(H * W * b) // 32)
        return a16(a16(a16(4 * P * WPP) + 8 * P) + es * P * (-(-H // B)) * (-(-W // B)))
    cases = [(2, 16, 32, 32, 8, 2, 4), (64, 256, 56, 56, 8, 2, 4), (64, 2048, 7, 7, 8, 2, 4), (3, 5, 55, 55, 4, 4, 4),
             (256, 256, 56, 56, 8, 2, 2), (1, 1, 1, 1, 1, 2, 4), (7, 3, 13, 29, 5, 4, 2),
             (64, 256, 56, 56, 8, 8, 4), (5, 3, 7, 7, 8, 8, 2), (3, 5, 7, 9, 4, 1, 4), (2, 2, 56, 56, 8, 1, 2)]
    for N, C, H, W, B, b, es in cases:
        dt = oracle.BF16 if es == 2 else oracle.F32
        assert oracle.packed_bytes(N, C, H, W, B, b, dt) == closed(N, C, H, W, B, b, es)
    assert oracle.packed_bytes(2, 16, 32, 32, 8, 2) == 10496
    # per-plane sizes of the ResNet-50 shapes: codes + 8 B meta + fp32 LFC
    for hw, total in [(112, 3928), (56, 988), (28, 268), (14, 76), (7, 28)]:
        lay = oracle.packed_layout(16, 1, hw, hw, 8, 2)
        assert (lay["codes_bytes"] + lay["meta_bytes"] + lay["lfc_bytes"]) // 16 == total
    for bad in [(0, 1, 4, 4, 2, 2), (1, 1, 4, 4, 0, 2), (1, 1, 4, 4, 2, 3), (1, 1, 4, 4, 2, 0), (1, 1, 4, 4, 2, 16)]:
        assert oracle.packed_bytes(*bad) == 0


def test_element_counts_reproduce_the_papers_accounting():
    pv = _paper_values()
    # LFC share at B=8 with the paper's bf16 LFC: LFC elements * 2 B / (4 B * map elements)
    lay = oracle.packed_layout(1, 1, 56, 56, 8, 2)
    n_lfc = lay["lfc_bytes"] // 4
    assert round(100 * n_lfc * 2 / (4 * 56 * 56), 1) == float(pv["lfc_share_B8_percent"])
    # HFC share at Q=2, N=7 with the paper's 4 B of (Delta, delta): (N^2 Q/8 + 4) / 4N^2
    N, Q = 7, 2
    code_bits = N * N * Q
    lay7 = oracle.packed_layout(1, 1, 7, 7, 8, 2)
    assert lay7["codes_bytes"] == 4 * -(-code_bits // 32)          # our codes are the same bits, word padded
    assert round(100 * (code_bits / 8 + 4) / (4 * N * N), 1) == float(pv["hfc_share_Q2_percent"])
    assert round(4 * N * N / (code_bits / 8 + 4)) == int(pv["hfc_only_rate"])
    # Theorem 3A from this layout's element counts (bf16 LFC, 4 B meta, 1-bit ReLU mask as in its proof)
    def rate(N, B, Q):
        lay = oracle.packed_layout(1, 1, N, N, B, Q)
        lfc_el = lay["lfc_bytes"] // 4
        ours = (2 * lfc_el + N * N * Q / 8 + 4) * 2 + N * N / 8
        return (4 * N * N * 2 + N * N) / ours
    formula = lambda N, B, Q: 9 / (4 / min(B * B, N * N) + Q / 4 + 8 / (N * N) + 1 / 8)
    for N in (7, 8, 16, 56, 112):          # B | N or N < B: the paper's own cases
        assert rate(N, 8, 2) == pytest.approx(formula(N, 8, 2), rel=1e-12)
    assert rate(7, 8, 2) == pytest.approx(10.346, abs=5e-4)
    assert round(rate(7, 8, 2), 2) == float(pv["theorem3A_min_rate"])
    assert all(rate(N, 8, 2) >= rate(7, 8, 2) for N in (8, 16, 56, 112))


# ---------------------------------------------------------------- R1..R3 random source

def test_hash_known_answers_independent_bigint():
    cases = [(0, 0, 0), (0, 0, 1), (0, 1, 0), (1, 0, 0), (1 << 32, 0, 0), (0xDEADBEEFCAFEF00D, 12345, 6789),
             (2 ** 64 - 1, 2 ** 31 - 1, 2 ** 31 - 1), (2, 970751, 6271), (0x0000000200000010, 77, 1567),
             (42, 3, 2 ** 24), (7, 2 ** 20, 2 ** 16 + 1), (0x123456789ABCDEF0, 1, 1)]
    got = [oracle.hash32(*c) for c in cases]
    assert got == [pyref.hash32(*c) for c in cases]
    frozen = {}
    with open(os.path.join(GOLDEN, "hash_kat.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].split()
            if len(line) == 4:
                frozen[tuple(int(v, 0) for v in line[:3])] = int(line[3], 0)
    assert len(frozen) >= 12
    for c, w in frozen.items():
        assert oracle.hash32(*c) == w and pyref.hash32(*c) == w
    for i in range(8):
        w = oracle.hash32(5, 9, i >> 1)
        assert oracle.rand16(5, 9, i) == ((w >> 16) if i & 1 else (w & 0xFFFF))


def test_hash_avalanche():
    rng = _rng(12)
    n = 1 << 14
    seeds = rng.integers(0, 2 ** 63, n, dtype=np.int64).astype(np.uint64)
    planes = rng.integers(0, 2 ** 31, n, dtype=np.int64)
    js = rng.integers(0, 2 ** 31, n, dtype=np.int64)
    base = np.array([pyref.hash32(int(s), int(p), int(j)) for s, p, j in zip(seeds, planes, js)], np.uint32)
    assert base.tolist()[:64] == [oracle.hash32(int(s), int(p), int(j)) for s, p, j in zip(seeds[:64], planes[:64], js[:64])]

    def flips(which, bit):
        out = np.empty(n, np.uint32)
        for k in range(n):
            s, p, j = int(seeds[k]), int(planes[k]), int(js[k])
            if which == 0:
                s ^= 1 << bit
            elif which == 1:
                p ^= 1 << bit
            else:
                j ^= 1 << bit
            out[k] = oracle.hash32(s, p, j)
        d = out ^ base
        return np.array([((d >> o) & 1).mean() for o in range(32)])

    for which, bits in ((0, (0, 1, 17, 31, 32, 47, 63)), (1, (0, 5, 19, 30)), (2, (0, 1, 2, 9, 23, 30))):
        for bit in bits:
            pr = flips(which, bit)
            assert np.all(np.abs(pr - 0.5) < 0.03), (which, bit, pr)


def test_hash_stream_statistics():
    n = 1 << 22
    w = oracle.hash32_fill(2, 1234, 0, n)
    lo, hi = (w & 0xFFFF).astype(np.float64), (w >> 16).astype(np.float64)
    for half in (lo, hi):
        assert abs(half.mean() - 32767.5) < 4.5 * 65536 / math.sqrt(12 * n)
        counts = np.bincount((half.astype(np.int64) >> 8), minlength=256)
        chi2 = ((counts - n / 256) ** 2 / (n / 256)).sum()
        assert chi2 < 255 + 4.5 * math.sqrt(2 * 255)                  # ~ 99.99 % band
        c = np.corrcoef(half[:-1], half[1:])[0, 1]
        assert abs(c) < 4.5 / math.sqrt(n)
    assert abs(np.corrcoef(lo, hi)[0, 1]) < 4.5 / math.sqrt(n)
    # low byte of each half is uniform as well (it decides rounding for tiny fractions)
    counts = np.bincount((w & 0xFF).astype(np.int64), minlength=256)
    assert ((counts - n / 256) ** 2 / (n / 256)).sum() < 255 + 4.5 * math.sqrt(2 * 255)
    # streams of neighbouring planes and neighbouring seeds are unrelated
    w2 = oracle.hash32_fill(2, 1235, 0, n)
    w3 = oracle.hash32_fill(3, 1234, 0, n)
    for other in (w2, w3):
        assert abs(np.corrcoef(w.astype(np.float64), other.astype(np.float64))[0, 1]) < 4.5 / math.sqrt(n)
        assert (w == other).mean() < 1e-5


# ---------------------------------------------------------------- planted mistakes are caught

def test_pins_would_catch_a_transposed_or_floor_pooled_oracle():
    # floor-mode pooling (dropping the ragged edge) and a transposed window
    # both disagree with the oracle on a ragged, non-square map
    x = _rng(13).standard_normal((1, 1, 6, 10)).astype(np.float32)
    p = oracle.compress(x, 4, 2, 0)
    lfc = oracle.split_packed(p, x.shape, 4, 2)["lfc"][0]
    assert lfc.shape == (2, 3)
    floor_mode = F.avg_pool2d(torch.from_numpy(x).double(), 4, 4).float().numpy()[0, 0]
    assert floor_mode.shape == (1, 2)
    assert np.array_equal(lfc[:1, :2], floor_mode)                    # interior windows agree
    xt = np.ascontiguousarray(x.transpose(0, 1, 3, 2))
    lfc_t = oracle.split_packed(oracle.compress(xt, 4, 2, 0), xt.shape, 4, 2)["lfc"][0]
    assert np.array_equal(lfc_t, lfc.T)


# ---------------------------------------------------------------- signed zeros

@pytest.mark.parametrize("dt", [oracle.F32, oracle.F32_C16])
def test_minimum_of_signed_zeros_does_not_depend_on_element_order(dt):
    # Eq. (quantization): delta = min H^H.  With +0 and -0 both present the reading is IEEE 754-2019 minimum:
    # -0, wherever it stands in the plane.  One block per plane with mean +0 keeps h = x.
    import itertools
    base = [0.0, -0.0, 0.0, -0.0]
    metas = set()
    for perm in set(itertools.permutations(base)):
        x = np.array(perm, dtype=np.float32).reshape(1, 1, 2, 2)
        s = oracle.split_packed(oracle.compress(x, 4, 2, 1, dt), x.shape, 4, 2, dt)
        metas.add(s["meta"].tobytes())
        assert s["lfc"].view(np.uint32 if dt == oracle.F32 else np.uint16).ravel()[0] == 0      # the mean is +0
    neg_zero = np.float32(-0.0).tobytes()
    want = neg_zero + np.float32(0).tobytes() if dt == oracle.F32 else neg_zero[2:] + b"\0\0"
    assert metas == {want}
    # blocks of one element: the mean of -0 is +0 (a sum that starts at 0), so h = x - mean is -0 exactly where
    # x is, +0 elsewhere; delta is -0 for every order of the elements, and the round trip gives +0 and 0.75
    for perm in set(itertools.permutations([0.0, -0.0, 0.75, -0.0])):
        x = np.array(perm, dtype=np.float32).reshape(1, 1, 1, 4)
        p = oracle.compress(x, 1, 2, 1, dt)
        s = oracle.split_packed(p, x.shape, 1, 2, dt)
        assert s["meta"].tobytes() == want
        assert oracle.decompress(p, x.shape, 1, 2, dt).tobytes() == np.abs(x).tobytes()


def test_block_mean_in_the_subnormal_range_rounds_ties_to_even():
    # Sec. 4.1 average pooling: exact sum / count, one rounding to binary32.  With elements k * 2^-149 the mean is
    # (sum k / count) * 2^-149, and binary32 keeps whole multiples of 2^-149 there: the rounding is that of a rational
    # to an integer, ties to even (python's round on a Fraction)
    from fractions import Fraction
    rng = _rng(41)
    tiny = 2.0 ** -149
    for cnt, shape, B in ((6, (1, 1, 2, 3), 4), (98, (1, 1, 7, 14), 16), (198, (1, 1, 11, 18), 18), (10, (1, 1, 1, 10), 16)):
        ties = 0
        for _ in range(300):
            k = rng.integers(-3000, 3000, cnt)
            if rng.random() < 0.5:                               # force an exact tie
                k[0] += (cnt // 2 - int(k.sum())) % cnt
            x = (k.astype(np.float64) * tiny).astype(np.float32).reshape(shape)
            assert np.array_equal(x.astype(np.float64).ravel() / tiny, k)
            lfc = oracle.split_packed(oracle.compress(x, B, 2, 3), shape, B, 2)["lfc"].ravel()
            want = round(Fraction(int(k.sum()), cnt))
            ties += (2 * int(k.sum())) % cnt == 0 and (2 * int(k.sum()) // cnt) % 2 == 1
            assert lfc.size == 1 and float(lfc[0]) / tiny == want
        assert ties > 100
