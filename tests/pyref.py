"""A second, deliberately different formulation of the codec for brute-force
pins on tiny inputs: exact rational arithmetic (fractions.Fraction) with an
explicit correctly-rounded conversion to binary32 after every fp32 step, a
per-element window search for the block mean, and a Python big-integer
evaluation of the random source.  Written from the paper's definitions
(Sec. 4.1, Sec. 4.2, Eq. (quantization)) and this build's stated readings;
it shares no code with the C oracle or with the GPU library.
"""
from fractions import Fraction
import math
import struct

M32 = 0xFFFFFFFF


def f32(fr: Fraction) -> Fraction:
    """Nearest binary32 value (ties to even) of an exact rational, as a Fraction."""
    if fr == 0:
        return Fraction(0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = math.floor(math.log2(a)) if a >= 1 else -math.ceil(math.log2(1 / a))
    # fix possible off-by-one of the float log
    while Fraction(2) ** e > a:
        e -= 1
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, -126)                      # subnormal range shares the exponent -126
    ulp = Fraction(2) ** (e - 23)
    n = a / ulp                           # exact rational number of ulps
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return sign * lo * ulp


def to_float(fr: Fraction) -> float:
    return float(fr)


def f32_next_up(fr: Fraction) -> Fraction:
    """Next binary32 above a positive binary32 value."""
    bits = struct.unpack("<I", struct.pack("<f", float(fr)))[0]
    return Fraction(struct.unpack("<f", struct.pack("<I", bits + 1))[0])


def mix32(x: int) -> int:
    x &= M32
    x ^= x >> 16
    x = (x * 0x7FEB352D) & M32
    x ^= x >> 15
    x = (x * 0x846CA68B) & M32
    x ^= x >> 16
    return x


def hash32(seed: int, plane: int, j: int) -> int:
    a = mix32((seed & M32) ^ 0x243F6A88)
    c = mix32(((seed >> 32) & M32) ^ 0x85A308D3)
    k1 = mix32(plane ^ a)
    k2 = mix32((k1 + c) & M32)
    x = (k1 + j * 0x9E3779B9) & M32
    x ^= x >> 16
    x = (x * 0x7FEB352D) & M32
    x = x ^ (x >> 15) ^ k2
    x = (x * 0x846CA68B) & M32
    x ^= x >> 16
    return x


def rand16(seed: int, plane: int, i: int) -> int:
    w = hash32(seed, plane, i >> 1)
    return (w >> 16) if (i & 1) else (w & 0xFFFF)


def bf16_floor(fr: Fraction) -> Fraction:
    """largest bfloat16 value <= fr (8 significant bits, binary32 exponent range; normal range only)"""
    if fr == 0:
        return Fraction(0)
    e = math.floor(math.log2(abs(fr)))
    while Fraction(2) ** e > abs(fr):
        e -= 1
    while Fraction(2) ** (e + 1) <= abs(fr):
        e += 1
    ulp = Fraction(2) ** (e - 7)
    return math.floor(fr / ulp) * ulp


def bf16_ceil(fr: Fraction) -> Fraction:
    return -bf16_floor(-fr)


def bf16_nearest(fr: Fraction) -> Fraction:
    lo, hi = bf16_floor(fr), bf16_ceil(fr)
    if lo == hi:
        return lo
    if fr - lo != hi - fr:
        return lo if fr - lo < hi - fr else hi
    # tie: even mantissa
    ulp = hi - lo
    return lo if (lo / ulp) % 2 == 0 else hi


def _range_is_usable(rng: Fraction) -> bool:
    """Reading of the degenerate plane (Eq. (quantization) divides by the range): a plane is
    quantised only if its rounded residual range is at least 2^-90 and is a finite binary32
    number.  A difference of two finite binary32 values whose nearest binary32 would need the
    exponent 128 has overflowed: f32() above returns 2^128 or more for it."""
    return Fraction(2) ** -90 <= rng < Fraction(2) ** 128


def codec_plane(x, H, W, B, b, seed, plane, c16=False):
    """x: list of H*W Fractions (exact binary32 values), row-major.
    c16: H^L, delta and Delta cached as bfloat16 (delta rounded down, Delta rounded up).

    Returns dict(lfc=[..], delta, Delta, codes=[..], xhat=[..]) with Fractions / ints.
    The block mean of an element is found by searching, per element, all
    elements that fall in the same B-aligned window (no block loop).
    """
    L = (1 << b) - 1
    LH, LW = -(-H // B), -(-W // B)
    mean_of = {}
    for r in range(H):
        for c in range(W):
            key = (r // B, c // B)
            if key in mean_of:
                continue
            members = [x[rr * W + cc] for rr in range(H) for cc in range(W)
                       if rr // B == key[0] and cc // B == key[1]]
            mean_of[key] = f32(sum(members, Fraction(0)) / len(members))
            if c16:
                mean_of[key] = bf16_nearest(mean_of[key])
    lfc = [mean_of[(i, j)] for i in range(LH) for j in range(LW)]
    h = [f32(x[r * W + c] - mean_of[(r // B, c // B)]) for r in range(H) for c in range(W)]
    delta, hmax = min(h), max(h)
    if c16:
        delta = bf16_floor(delta)
    rng = f32(hmax - delta)
    usable = _range_is_usable(rng)
    if usable and c16 and bf16_ceil(f32(rng / L)) >= Fraction(2) ** 128:
        usable = False               # the step has no finite bfloat16 to be cached as (1-bit codes only)
    if usable and c16:
        Delta = bf16_ceil(f32(rng / L))
        inv = f32(1 / Delta)
    elif usable:
        Delta = f32(rng / L)
        inv = f32(Fraction(L) / rng)
        if f32(rng * inv) < L:
            inv = f32_next_up(inv)
    else:
        Delta = inv = Fraction(0)
    codes, xhat = [], []
    for i, hv in enumerate(h):
        t = f32(f32(hv - delta) * inv)
        q = min(L, math.floor(t + Fraction(rand16(seed, plane, i), 65536)))
        codes.append(q)
        hh = f32(f32(q * Delta) + delta)
        xhat.append(f32(mean_of[(i // W // B, i % W // B)] + hh))
    return {"lfc": lfc, "delta": delta, "Delta": Delta, "codes": codes, "xhat": xhat, "h": h}


def codec_volume(x, dims, B, b, seed, plane):
    """Exact-rational codec of one plane with any number of map dimensions (Appendix D: 1-D, 2-D
    and 3-D maps share one definition).  x: list of prod(dims) Fractions in row-major order.
    The block of an element is the tuple of its coordinates floor-divided by B; the members of a
    block are found by a search over all elements (no block loop)."""
    L = (1 << b) - 1
    n = len(x)
    coords = []
    for i in range(n):
        c, rem = [], i
        for d in reversed(dims):
            c.append(rem % d)
            rem //= d
        coords.append(tuple(reversed(c)))
    key = [tuple(v // B for v in c) for c in coords]
    mean_of = {}
    for k in sorted(set(key)):
        members = [x[i] for i in range(n) if key[i] == k]
        mean_of[k] = f32(sum(members, Fraction(0)) / len(members))
    lfc = [mean_of[k] for k in sorted(mean_of)]           # row-major order of the pooled map
    h = [f32(x[i] - mean_of[key[i]]) for i in range(n)]
    delta, hmax = min(h), max(h)
    rng = f32(hmax - delta)
    if _range_is_usable(rng):
        Delta = f32(rng / L)
        inv = f32(Fraction(L) / rng)
        if f32(rng * inv) < L:
            inv = f32_next_up(inv)
    else:
        Delta = inv = Fraction(0)
    codes, xhat = [], []
    for i, hv in enumerate(h):
        t = f32(f32(hv - delta) * inv)
        q = min(L, math.floor(t + Fraction(rand16(seed, plane, i), 65536)))
        codes.append(q)
        xhat.append(f32(mean_of[key[i]] + f32(f32(q * Delta) + delta)))
    return {"lfc": lfc, "delta": delta, "Delta": Delta, "codes": codes, "xhat": xhat, "h": h}
