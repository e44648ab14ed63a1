"""Pins of the oracle's roundings (no GPU): places where a plausible slip changes a result only once in
tens of thousands of elements, so that random inputs do not see it.

* Eq. (quantization), stochastic rounding: code = floor(t + u) with u = r / 2^16 uniform on
  {0, 1/65536, ..., 65535/65536}.  The planes below are built so that, for the random bits the element
  really gets, t + u is exactly an integer, one step of u below an integer, or 2^-25 below an integer;
  delta, Delta, H^L and the scale are exact powers of two by construction, so every expected code is
  derived by hand.  A generator shifted by one step (u in (0, 1]), a sum formed in binary32, or a scale
  that is bumped although L / range is exact each move one of these codes.
* bfloat16 storage (Sec. 4.1 caches H^L in bfloat16; a bfloat16 map is rebuilt in bfloat16): conversion is
  round-to-nearest-even, NaN stays NaN.  Checked against torch's conversion (a library routine) and
  against values worked out by hand, on the conversion itself and on a hand-made packed buffer.
"""
import numpy as np
import pytest
import torch

import oracle

TWO16 = 65536


def _tie_plane(seed, b=2):
    """A 128 x 128 plane that is one block (B = 128), built backwards from the codes it must give.

    Residual = the value itself (the block sum is exactly zero, so H^L = +0).  delta = -2^-16,
    max = 3 * 2^-10 - 2^-16, hence range = L * 2^-10 with L = 3, Delta = 2^-10, scale = 2^10 exactly
    (range * scale == L: no correction of the scale), and t = (h + 2^-16) * 2^10 without rounding for
    the values used.  Returns x, and {index: expected code} for the constructed elements."""
    assert b == 2
    HW = 128 * 128
    delta = -2.0 ** -16
    x = np.zeros(HW, dtype=np.float64)
    expect = {}
    x[0] = 3 * 2.0 ** -10 + delta                  # the maximum: t = 3 -> top code for any u
    expect[0] = 3
    kinds = 0
    i = 1
    want = {"integer": 12, "step_below": 12, "sub_ulp": 12}
    while any(want.values()) and i < 4000:
        r = oracle.rand16(seed, 0, i)
        t = None
        if want["integer"] and 1 <= r:
            k = want["integer"] % 2                # t + u == k + 1 exactly -> code k + 1
            t = k + (TWO16 - r) / TWO16
            code = k + 1
            want["integer"] -= 1
        elif want["step_below"] and r <= TWO16 - 2:
            k = want["step_below"] % 2             # t + u == k + 1 - 2^-16 -> code k
            t = k + (TWO16 - r - 1) / TWO16
            code = k
            want["step_below"] -= 1
        elif want["sub_ulp"] and TWO16 // 2 <= r <= 3 * TWO16 // 4:
            t = (TWO16 - r) / TWO16 - 2.0 ** -25   # t + u == 1 - 2^-25: below 1 -> code 0; t in [0.25, 0.5)
            code = 0
            want["sub_ulp"] -= 1
        if t is not None:
            h = t * 2.0 ** -10 + delta
            assert float(np.float32(h)) == h       # representable: nothing is rounded on the way in
            x[i] = h
            expect[i] = code
            kinds += 1
        i += 1
    assert not any(want.values())
    # fillers in [delta, 0] that bring the block sum to exactly zero (all values are multiples of 2^-35,
    # the partial sums stay far below 2^53 of them: the binary64 sum is exact in any order)
    need = x.sum()
    assert need > 0
    free = [j for j in range(4000, HW)]
    n_full = int(need // -delta)
    rest = need - n_full * -delta
    assert n_full + 1 < len(free)
    for j in free[:n_full]:
        x[j] = delta
        expect[j] = 0                              # the minimum: t = 0, code 0 for any u < 1
    x[free[n_full]] = -rest
    assert float(np.float32(rest)) == rest
    assert x.sum() == 0.0 and x.min() == delta
    return x.astype(np.float32).reshape(1, 1, 128, 128), expect


@pytest.mark.parametrize("seed", [1, 0xC0FFEE, 2 ** 63 + 5])
def test_codes_on_exact_ties_of_the_stochastic_rounding(seed):
    x, expect = _tie_plane(seed)
    p, dbg = oracle.compress(x, 128, 2, seed, oracle.F32, debug=True)
    s = oracle.split_packed(p, x.shape, 128, 2, oracle.F32)
    assert s["lfc"].view(np.uint32).tolist() == [[[0]]]                     # H^L = +0
    assert s["meta"][0, 0] == np.float32(-2.0 ** -16) and s["meta"][0, 1] == np.float32(2.0 ** -10)
    q = oracle.unpack_codes(s["codes"], 128 * 128, 2)[0]
    t = dbg["t"].reshape(-1)
    assert t[0] == np.float32(3.0)
    bad = [(i, int(q[i]), c, float(t[i]), oracle.rand16(seed, 0, i)) for i, c in expect.items() if int(q[i]) != c]
    assert not bad, bad[:5]
    # and the decoder's side of the same plane: Delta * code + delta on top of H^L = 0
    y = oracle.decompress(p, x.shape, 128, 2, oracle.F32).reshape(-1)
    for i, c in list(expect.items())[:64]:
        assert y[i] == np.float32(c * 2.0 ** -10 - 2.0 ** -16)


def tie_map(shape, seed, B=8):
    """The same construction for maps of many B x B blocks (b = 2): every block's sum is exactly zero, so
    H^L = +0 everywhere and the residual is the value; per plane delta = -2^-12 and max = 3 * 2^-10 - 2^-12,
    so Delta = 2^-10 and the scale is 2^10 without correction.  The first element of every block is built
    from its own random bits r so that t + u is exactly 1, one step of u below 1, or 2^-25 below 1; the
    rest of the block are fillers in [delta, 0] that cancel it.  Returns x and, per plane, {index: code}."""
    N, C, H, W = shape
    delta = -2.0 ** -12
    x = np.zeros((N * C, H, W), dtype=np.float64)
    expect = [dict() for _ in range(N * C)]
    for p in range(N * C):
        first = True
        for r0 in range(0, H, B):
            for c0 in range(0, W, B):
                cells = [(r, c) for r in range(r0, min(H, r0 + B)) for c in range(c0, min(W, c0 + B))]
                if len(cells) < 16:
                    continue                              # a sliver of a block: left at zero
                (tr, tc), fill = cells[0], cells[1:]
                i = tr * W + tc
                r16 = oracle.rand16(seed, p, i)
                if first:
                    h, code = 3 * 2.0 ** -10 + delta, 3   # the plane's maximum: t = 3
                    first = False
                elif TWO16 // 2 <= r16 <= 3 * TWO16 // 4:
                    h, code = ((TWO16 - r16) / TWO16 - 2.0 ** -25) * 2.0 ** -10 + delta, 0
                elif r16 >= 1 and (i // B) % 2 == 0:
                    h, code = ((TWO16 - r16) / TWO16) * 2.0 ** -10 + delta, 1
                elif r16 <= TWO16 - 2:
                    h, code = ((TWO16 - r16 - 1) / TWO16) * 2.0 ** -10 + delta, 0
                else:
                    h, code = 0.0, None
                assert float(np.float32(h)) == h
                x[p, tr, tc] = h
                if code is not None:
                    expect[p][i] = code
                # cancel h with fillers in [delta, 0]
                need = h
                if need < 0:
                    x[p, fill[0][0], fill[0][1]] = -need  # a positive filler below the maximum
                    need = 0.0
                n_full = int(need // -delta)
                rest = need - n_full * -delta
                assert n_full + 1 < len(fill) and float(np.float32(rest)) == rest
                for (fr, fc) in fill[1:1 + n_full]:
                    x[p, fr, fc] = delta
                    expect[p][fr * W + fc] = 0
                x[p, fill[1 + n_full][0], fill[1 + n_full][1]] = -rest
                assert sum(x[p, r, c] for (r, c) in cells) == 0.0
        assert x[p].min() == delta and x[p].max() == 3 * 2.0 ** -10 + delta
    return x.astype(np.float32).reshape(shape), expect


@pytest.mark.parametrize("shape", [(2, 3, 56, 56), (2, 2, 28, 28), (3, 2, 14, 14), (2, 2, 24, 40)])
def test_codes_on_exact_ties_in_maps_of_many_blocks(shape):
    seed = 0xBEEF
    x, expect = tie_map(shape, seed)
    p = oracle.compress(x, 8, 2, seed, oracle.F32)
    s = oracle.split_packed(p, shape, 8, 2, oracle.F32)
    assert not s["lfc"].view(np.uint32).any()                               # every H^L is +0
    assert np.all(s["meta"][:, 0] == np.float32(-2.0 ** -12)) and np.all(s["meta"][:, 1] == np.float32(2.0 ** -10))
    q = oracle.unpack_codes(s["codes"], shape[2] * shape[3], 2)
    kinds = set()
    for pl, e in enumerate(expect):
        assert len(e) > 4
        for i, c in e.items():
            assert int(q[pl, i]) == c, (pl, i, int(q[pl, i]), c, oracle.rand16(seed, pl, i))
            kinds.add(c)
    assert kinds == {0, 1, 3}


def _bits_of(f32_array):
    return np.array([oracle.lib().oracle_float_to_bf16(float(v)) for v in f32_array], dtype=np.uint16)


def test_bfloat16_conversion_rounds_to_nearest_even_by_hand():
    cases = [
        (1.0 + 2.0 ** -8, 0x3F80),                 # halfway between 1 and 1 + 2^-7: to the even one, down
        (1.0 + 3 * 2.0 ** -8, 0x3F82),             # halfway between 0x3F81 and 0x3F82: to the even one, up
        (1.0 + 2.0 ** -8 + 2.0 ** -23, 0x3F81),    # just above halfway
        (1.0 + 2.0 ** -8 - 2.0 ** -23, 0x3F80),    # just below halfway
        (-(1.0 + 2.0 ** -8), 0xBF80),
        (-(1.0 + 3 * 2.0 ** -8), 0xBF82),
        (float(np.finfo(np.float32).max), 0x7F80), # rounds up to infinity
        (2.0 ** -133, 0x0001),                     # smallest subnormal bfloat16, exact
        (2.0 ** -134, 0x0000),                     # halfway between 0 and it: to even, zero
        (3 * 2.0 ** -134, 0x0002),                 # halfway between 1 and 2 steps: to even
        (0.0, 0x0000), (-0.0, 0x8000), (float("inf"), 0x7F80), (float("-inf"), 0xFF80),
    ]
    for v, want in cases:
        assert int(oracle.lib().oracle_float_to_bf16(v)) == want, (v, hex(want))


def test_bfloat16_conversion_agrees_with_the_library_conversion():
    rng = np.random.default_rng(5)
    bits = rng.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32)
    # every kind of tie and near-tie in the low half
    ties = (rng.integers(0, 2 ** 16, size=20000, dtype=np.uint64).astype(np.uint32) << 16) | np.uint32(0x8000)
    near = np.concatenate([ties + np.uint32(1), ties - np.uint32(1)])
    v = np.concatenate([bits, ties, near]).view(np.float32)
    finite = np.isfinite(v)
    lib_bits = torch.from_numpy(v.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    mine = _bits_of(v[::7])                        # the scalar call is slow from Python: every 7th value
    assert np.array_equal(mine[finite[::7]], lib_bits[::7][finite[::7]])
    assert np.array_equal(oracle.bf16_bits(v[finite]), lib_bits[finite])


def test_bfloat16_conversion_keeps_nan():
    for pattern in (0x7F800001, 0x7F80FFFF, 0x7FC00000, 0xFF800001, 0x7FFFFFFF, 0x7F808000):
        f = np.array([pattern], dtype=np.uint32).view(np.float32)[0]
        out = int(oracle.lib().oracle_float_to_bf16(float(f)))
        assert (out & 0x7FFF) > 0x7F80, hex(pattern)           # still a NaN, not an infinity
        assert (out >> 15) == (pattern >> 31)


def test_bfloat16_map_is_rebuilt_with_round_to_nearest_even():
    # a hand-made packed buffer: one plane of 8 elements, one block, 8-bit codes; H^L = 1, delta = 0,
    # Delta = 2^-9, so xhat = 1 + code * 2^-9 rounded to bfloat16 (spacing 2^-7 above 1)
    shape, B, b = (1, 1, 1, 8), 8, 8
    p = np.zeros(oracle.packed_bytes(*shape, B, b, oracle.BF16), dtype=np.uint8)
    s = oracle.split_packed(p, shape, B, b, oracle.BF16)
    codes = [0, 1, 2, 3, 4, 5, 6, 7]
    s["codes"][0, 0] = sum(c << (8 * i) for i, c in enumerate(codes[:4]))
    s["codes"][0, 1] = sum(c << (8 * i) for i, c in enumerate(codes[4:]))
    s["meta"][0, 0] = 0.0
    s["meta"][0, 1] = 2.0 ** -9
    s["lfc"][0, 0, 0] = 0x3F80
    y = oracle.decompress(p, shape, B, b, oracle.BF16).reshape(-1)
    #        1      +1/4 step  tie->even(down)  above tie  one step  +1/4      tie->even(up)  above
    want = [0x3F80, 0x3F80,    0x3F80,          0x3F81,    0x3F81,   0x3F81,   0x3F82,        0x3F82]
    assert [int(v) for v in y] == want
    lib_bits = torch.tensor([1 + c * 2.0 ** -9 for c in codes], dtype=torch.float32).to(torch.bfloat16).view(torch.int16)
    assert [int(v) & 0xFFFF for v in lib_bits] == want
