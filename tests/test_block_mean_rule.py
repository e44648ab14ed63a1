"""The block mean of Sec. 4.1 (AveragePooling) as the compress kernels evaluate it, checked on the host.

Definition (what the oracle computes): mean = (float)(S / cnt), S the exact sum of the block in binary64,
one binary64 division, one rounding to binary32.  The kernels multiply by the reciprocal and divide only
when the product is close to a rounding boundary of binary32 or below the smallest normal binary32.
`division_block_mean_rule` runs that rule's source on the host; here it has to agree with the definition
(numpy's IEEE division and conversion, and exact rationals for the placed cases) for every block count a
kernel can meet, on sums placed on and right beside every kind of rounding boundary.  No GPU needed.
"""
import ctypes
from fractions import Fraction

import numpy as np
import pytest

import paper_2208_04187_amd as pkg


def _rule():
    L = pkg.lib()
    f = L.division_block_mean_rule
    f.restype = ctypes.c_float
    f.argtypes = [ctypes.c_double, ctypes.c_uint32, ctypes.POINTER(ctypes.c_int)]
    return f


def _definition(S: np.ndarray, cnt: int) -> np.ndarray:
    with np.errstate(over="ignore"):          # a quotient beyond binary32 is +-inf on both sides
        return (S.astype(np.float64) / np.float64(cnt)).astype(np.float32)


def _check(rule, S: np.ndarray, cnt: int, tally):
    want = _definition(S, cnt)
    d = ctypes.c_int(0)
    for s, w in zip(S.tolist(), want):
        got = np.float32(rule(s, cnt, ctypes.byref(d)))
        tally[0] += 1
        tally[1] += d.value
        assert got.view(np.uint32) == w.view(np.uint32), (cnt, float.hex(s), float(got), float(w))


def _beside(S: np.ndarray) -> np.ndarray:
    """S and the binary64 numbers 1, 2 and 3 ulp on either side of it."""
    out = [S]
    up, dn = S, S
    for _ in range(3):
        up = np.nextafter(up, np.inf)
        dn = np.nextafter(dn, -np.inf)
        out += [up, dn]
    return np.concatenate(out)


def _placed_sums(cnt: int, rng) -> np.ndarray:
    """Sums whose exact quotient by cnt is a rounding boundary of binary32 (the midpoint of two
    neighbouring binary32 numbers), a binary32 number, or a hair beside either: normal results at a
    spread of exponents, results at both ends of the subnormal range, and the smallest normal."""
    sums = []
    # normal binary32 results: midpoint (2k+1) * 2^(e-24) and exact value 2k * 2^(e-24)
    for e in (-126, -125, -100, -24, -1, 0, 1, 23, 60, 96):
        k = rng.integers(1 << 23, 1 << 24, size=3)
        for odd in (1, 0):
            m = (2 * k + odd).astype(np.float64) * 2.0 ** (e - 24)
            sums.append(m * cnt)                               # exact: (2k+1)*cnt < 2^53
    # subnormal binary32 results: midpoints (j + 1/2) * 2^-149 and exact values j * 2^-149
    j = np.concatenate([np.arange(0, 6), rng.integers(6, 1 << 23, size=4), [(1 << 23) - 2, (1 << 23) - 1]])
    sums.append((2 * j + 1).astype(np.float64) * 2.0 ** -150 * cnt)
    sums.append(j.astype(np.float64) * 2.0 ** -149 * cnt)
    S = np.concatenate(sums)
    S = np.concatenate([S, -S[::3]])
    return _beside(S)


def test_placed_sums_are_what_they_claim():
    """The construction above really lands on ties: exact rationals for one count."""
    cnt = 98
    k = 0x923456
    S = float((2 * k + 1) * cnt) * 2.0 ** (-24 - 24)
    assert Fraction(S) / cnt == Fraction(2 * k + 1, 2 ** 48)                  # a midpoint of binary32 at exponent -24
    S = float(7 * cnt) * 2.0 ** -150
    assert Fraction(S) / cnt == Fraction(7, 2) * Fraction(1, 2 ** 149)        # 3.5 steps of the subnormal grid


def test_rule_equals_definition_for_every_count_up_to_4096():
    rule = _rule()
    rng = np.random.default_rng(2024)
    tally = [0, 0]
    for cnt in range(1, 4097):
        _check(rule, _placed_sums(cnt, rng), cnt, tally)
    # the division is the exception even on this adversarial set's exact values (ties always take it)
    assert tally[1] > 0 and tally[0] > 400000


def test_rule_equals_definition_for_large_and_awkward_counts():
    """Counts of 3-D blocks and whole planes (B^3, H*W for one-block planes), primes, numbers next to
    powers of two, the largest count the library admits."""
    rule = _rule()
    rng = np.random.default_rng(7)
    counts = [5 ** 3, 12 ** 3, 18 ** 3, 64 ** 3, 55 * 55, 147 * 147, 299 * 299, 4097, 65535, 65537, 1000003,
              (1 << 20) - 1, (1 << 20) + 1, (1 << 27) - 39]
    tally = [0, 0]
    for cnt in counts:
        _check(rule, _placed_sums(cnt, rng), cnt, tally)
    # beyond 2^28 the placed products no longer fit binary64 exactly: random sums there
    for cnt in [(1 << 31) - 1, (1 << 30) + 3, 3 * (1 << 29) + 1]:
        S = rng.standard_normal(4000) * 10.0 ** rng.uniform(-30, 30, 4000) * cnt
        _check(rule, S, cnt, tally)


def test_rule_equals_definition_on_random_sums_of_binary32_values():
    rule = _rule()
    rng = np.random.default_rng(99)
    tally = [0, 0]
    for cnt in (3, 6, 10, 36, 48, 49, 98, 150, 196, 198, 324, 3025):
        x = (rng.standard_normal((300, cnt)) * 10.0 ** rng.uniform(-42, 30, (300, 1))).astype(np.float32)
        S = x.astype(np.float64).sum(axis=1)
        _check(rule, S, cnt, tally)
    assert tally[1] < tally[0] // 10


def test_means_below_the_smallest_normal_take_the_division():
    """A nonzero mean that rounds to a subnormal binary32 must not use the reciprocal: for counts such as
    98 the product S * fl(1/98) sits one binary64 ulp beside an exact tie of the subnormal grid, and the
    29 low bits the rule inspects do not show it.  (3.5 steps -> 4 steps, ties to even.)"""
    rule = _rule()
    d = ctypes.c_int(0)
    for cnt in (6, 10, 98, 196, 198):
        S = float(7 * cnt) * 2.0 ** -150
        got = np.float32(rule(S, cnt, ctypes.byref(d)))
        assert d.value == 1
        assert got == np.float32(4 * 2.0 ** -149)
        S = float(5 * cnt) * 2.0 ** -150                                       # 2.5 steps -> 2 steps
        assert np.float32(rule(S, cnt, ctypes.byref(d))) == np.float32(2 * 2.0 ** -149)


def test_powers_of_two_never_divide_and_zero_count_is_zero():
    rule = _rule()
    d = ctypes.c_int(0)
    for cnt in (1, 2, 64, 4096, 1 << 30):
        assert np.float32(rule(3.0 * cnt, cnt, ctypes.byref(d))) == np.float32(3.0) and d.value == 0
    assert rule(5.0, 0, None) == 0.0
