"""Pins of the oracle's threshold edges (no GPU).

Eq. (quantization) divides by the residual range of a plane; the reading taken for planes where that
division cannot be done is: a plane is quantised iff its rounded residual range lies in
[2^-90, largest binary32], otherwise Delta = 0, every code is 0 and xhat = H^L + delta.  These tests
stand planes on both sides of each edge and state by hand what has to come out; the exact-rational
second formulation (tests/pyref.py) must agree element by element as well.

The Dropout operator keeps an element iff its 16 random bits r satisfy r >= T, T = round(p * 65536):
only then is the keep probability (65536 - T) / 65536 = 1 - p, the Bernoulli(1 - p) of the listing, and
only then does p = 0 keep everything.  The tests construct inputs on which some element has r == T.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from tests import pyref

C16 = oracle.F32_C16
TWO_M90 = np.float32(2.0 ** -90)
BELOW = np.nextafter(TWO_M90, np.float32(0))        # largest binary32 below 2^-90
ABOVE = np.nextafter(TWO_M90, np.float32(1))        # smallest binary32 above 2^-90
FLT_MAX = np.finfo(np.float32).max


def _meta_f32(s, dt):
    m = s["meta"]
    return oracle.bf16_to_f32(m) if dt == C16 else m


def _one_plane(values, H, W, B, b, dt, seed=7):
    x = np.asarray(values, dtype=np.float32).reshape(1, 1, H, W)
    p = oracle.compress(x, B, b, seed, dt)
    s = oracle.split_packed(p, x.shape, B, b, dt)
    q = oracle.unpack_codes(s["codes"], H * W, b)[0]
    xh = oracle.decompress(p, x.shape, B, b, dt).ravel()
    meta = _meta_f32(s, dt)
    ref = pyref.codec_plane([Fraction(float(v)) for v in x.ravel()], H, W, B, b, seed, 0, c16=(dt == C16))
    # the second formulation agrees on everything stored and rebuilt
    assert Fraction(float(meta[0, 0])) == ref["delta"]
    assert Fraction(float(meta[0, 1])) == ref["Delta"]
    assert q.tolist() == ref["codes"]
    assert [Fraction(float(v)) for v in xh] == ref["xhat"]
    return float(meta[0, 0]), float(meta[0, 1]), q, xh


# ---------------------------------------------------------------- lower edge: residual range around 2^-90

@pytest.mark.parametrize("dt", [oracle.F32, C16])
@pytest.mark.parametrize("b", [1, 2, 4, 8])
def test_residual_range_just_below_at_and_just_above_the_lower_edge(dt, b):
    """A 1 x 2 plane (0, v) under B = 2 is one block with mean v/2 (exact: a halving), so the
    residuals are -v/2 and v - v/2 and their range is v, up to the one rounding of the subtraction
    that the cases below avoid.  In the bfloat16-cached format the mean 2^-91 is a bfloat16 number
    for all three v (v/2 rounds to it), delta = -2^-91 needs no rounding, and the range is again a
    binary32 number next to 2^-90."""
    L = (1 << b) - 1
    # just below: degenerate
    delta, Delta, q, xh = _one_plane([0.0, BELOW], 1, 2, 2, b, dt)
    assert Delta == 0.0 and q.tolist() == [0, 0]
    if dt == oracle.F32:
        assert delta == -float(BELOW) / 2
        assert xh.tolist() == [0.0, 0.0]                         # H^L + delta = v/2 - v/2 for both elements
    else:
        assert delta == -(2.0 ** -91)
        assert xh.tolist() == [0.0, 0.0]
    # exactly 2^-90: quantised; the minimum takes code 0 and the maximum the top code for every seed
    for seed in range(5):
        delta, Delta, q, xh = _one_plane([0.0, TWO_M90], 1, 2, 2, b, dt, seed)
        assert delta == -(2.0 ** -91)
        if dt == oracle.F32:
            assert Delta == float(np.float32(TWO_M90) / np.float32(L))
        else:
            # fl(2^-90 / L) rounded up to 8 significant bits
            exact = Fraction(float(np.float32(TWO_M90) / np.float32(L)))
            assert Fraction(Delta) == pyref.bf16_ceil(exact) and Fraction(Delta) >= exact
        assert Delta > 0.0
        if dt == oracle.F32:
            assert q.tolist() == [0, L]
        else:
            assert q[0] == 0 and q[1] >= L - 1                  # Delta is rounded up: the top code need not be reached
        assert xh[0] == 0.0 and abs(xh[1] - float(TWO_M90)) <= Delta
    # just above: quantised
    delta, Delta, q, xh = _one_plane([0.0, ABOVE], 1, 2, 2, b, dt)
    assert Delta > 0.0 and q[0] == 0 and q[1] >= L - 1


@pytest.mark.parametrize("dt", [oracle.F32, C16])
def test_a_larger_plane_whose_range_sits_on_the_lower_edge(dt):
    """4 x 4, one block (B = 4), fifteen zeros and one element v: mean v/16 (exact), residuals -v/16
    and v - v/16 = 15v/16 (exact for v a power of two), range v.  v = 2^-90 is quantised, v = 2^-91
    is not."""
    for v, quantised in [(2.0 ** -90, True), (2.0 ** -91, False), (2.0 ** -89, True)]:
        vals = [0.0] * 16
        vals[5] = v
        delta, Delta, q, xh = _one_plane(vals, 4, 4, 4, 2, dt)
        assert delta == -v / 16
        if quantised:
            assert Delta > 0 and q[5] >= 2 and all(q[i] == 0 for i in range(16) if i != 5)
        else:
            assert Delta == 0 and not q.any()
            assert np.all(xh == 0.0)                             # H^L + delta = v/16 - v/16


# ---------------------------------------------------------------- upper edge: ranges beyond binary32

@pytest.mark.parametrize("dt", [oracle.F32, C16])
@pytest.mark.parametrize("b", [1, 2, 4])
def test_residual_range_that_overflows_binary32_is_degenerate(dt, b):
    """(-a, a) with a = 2^127 (a bfloat16 number too): mean 0, residuals -a and a, both finite, but
    a - (-a) = 2^128 is not a binary32 number.  The plane is not quantised: Delta = 0, codes 0,
    xhat = H^L + delta = -a for both elements."""
    a = 2.0 ** 127
    delta, Delta, q, xh = _one_plane([-a, a], 1, 2, 2, b, dt)
    assert delta == -a and Delta == 0.0
    assert q.tolist() == [0, 0]
    assert xh.tolist() == [-a, -a]


@pytest.mark.parametrize("b", [1, 2, 4])
def test_largest_finite_residual_range_is_still_quantised(b):
    """(-m/2, m/2) with m the largest binary32: the range is m itself, finite, so the plane is
    quantised: Delta = fl(m / L) > 0, the extremes take the end codes."""
    L = (1 << b) - 1
    m = float(FLT_MAX)
    delta, Delta, q, xh = _one_plane([-m / 2, m / 2], 1, 2, 2, b, oracle.F32)
    assert delta == -m / 2
    assert Delta == float(np.float32(FLT_MAX) / np.float32(L))
    assert q.tolist() == [0, L]
    assert xh[0] == -m / 2 and abs(xh[1] - m / 2) <= Delta


def test_largest_finite_residual_range_in_the_bfloat16_cached_format():
    """The same with values that are bfloat16 numbers: a = largest bfloat16 / 2; range = largest
    bfloat16 (finite), Delta = fl(range / 3) rounded up to bfloat16."""
    big = float(oracle.bf16_to_f32(np.array([0x7F7F], dtype=np.uint16))[0])
    delta, Delta, q, xh = _one_plane([-big / 2, big / 2], 1, 2, 2, 2, C16)
    assert delta == -big / 2 and Delta > 0 and q[0] == 0 and q[1] >= 2


def test_a_step_beyond_the_largest_bfloat16_makes_the_plane_degenerate_in_the_cached_format():
    """1-bit codes, bfloat16-cached tuple: (-a, a) with a = 1.99609375 * 2^126 (nine significant bits, not a
    bfloat16).  delta = -a rounded down to bfloat16 = -2^127, the range a + 2^127 = 1.998046875 * 2^127 is a finite
    binary32 number, but Delta = range / 1 rounded up to bfloat16 would be 2^128: there is no finite step to cache.
    The plane is not quantised: Delta = 0, codes 0, xhat = H^L + delta = -2^127 (finite, not NaN).  In the fp32
    format the same plane is quantised: Delta = 2a, codes 0 and 1, rebuilt exactly."""
    a = 1.99609375 * 2.0 ** 126
    delta, Delta, q, xh = _one_plane([-a, a], 1, 2, 2, 1, C16)
    assert delta == -(2.0 ** 127) and Delta == 0.0
    assert q.tolist() == [0, 0]
    assert xh.tolist() == [-(2.0 ** 127)] * 2 and np.isfinite(xh).all()
    delta, Delta, q, xh = _one_plane([-a, a], 1, 2, 2, 1, oracle.F32)
    assert delta == -a and Delta == 2 * a and q.tolist() == [0, 1] and xh.tolist() == [-a, a]


def test_the_largest_step_that_is_a_bfloat16_is_still_used():
    """1-bit codes, cached format: (-a, a) with a = 1.9921875 * 2^126 (a bfloat16): range = largest bfloat16 exactly,
    Delta = range, the extremes take codes 0 and 1 and are rebuilt exactly."""
    big = float(oracle.bf16_to_f32(np.array([0x7F7F], dtype=np.uint16))[0])
    delta, Delta, q, xh = _one_plane([-big / 2, big / 2], 1, 2, 2, 1, C16)
    assert delta == -big / 2 and Delta == big
    assert q.tolist() == [0, 1] and xh.tolist() == [-big / 2, big / 2]


# ---------------------------------------------------------------- Dropout: the element whose bits equal the threshold

def _dropout_stream(seed, n):
    s = seed ^ 0xD509A5B3C2E1F047
    return np.array([pyref.rand16(s, 0, i) for i in range(n)], dtype=np.int64)


def test_dropout_keeps_the_element_whose_random_bits_equal_the_threshold():
    n, seed = 4096, 0x5EED_0000_0000_0042
    r = _dropout_stream(seed, n)
    # a threshold that some element hits exactly, and that others miss by one on either side
    cands = [int(t) for t in np.unique(r) if 0 < t < 65536 and (r == t - 1).any() and (r == t + 1).any()]
    T = cands[len(cands) // 2] if cands else int(r[17])
    p = T / 65536.0                                              # a binary32 number: T has at most 16 bits
    assert oracle.dropout_threshold(p) == T
    x = np.arange(1, n + 1, dtype=np.float32)
    y, mask = oracle.dropout_forward(x, p, seed)
    bits = ((mask.view(np.uint32)[np.arange(n) // 32] >> (np.arange(n) % 32)) & 1).astype(bool)
    assert (r == T).any()
    assert bits[r == T].all()                                    # r == T is kept ...
    assert not bits[r == T - 1].any()                            # ... r == T - 1 is dropped
    assert np.array_equal(bits, r >= T)
    assert np.array_equal(y, np.where(r >= T, x, np.float32(0)))
    # the keep probability over all 2^16 values of r is then exactly 1 - p
    assert Fraction(int((np.arange(65536) >= T).sum()), 65536) == 1 - Fraction(p)


def test_dropout_with_p_zero_keeps_an_element_whose_random_bits_are_all_zero():
    """Bernoulli(1 - 0) keeps every element (listing of the Dropout operator).  The stream of this
    seed holds an element with r = 0 among its first 2^18; it has to be kept."""
    seed = 3
    n = 1 << 18
    r = _dropout_stream(seed, n)
    zeros = np.flatnonzero(r == 0)
    assert zeros.size > 0
    n = int(zeros[0]) + 33
    x = np.full(n, 2.5, dtype=np.float32)
    y, mask = oracle.dropout_forward(x, 0.0, seed)
    assert np.all(y == 2.5)
    assert int(sum(bin(int(w)).count("1") for w in mask.view(np.uint32))) == n
