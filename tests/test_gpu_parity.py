"""GPU parity: the HIP library (through its C ABI) against the CPU oracle,
element by element on the same seeded inputs.  Needs a real MI355X."""
import numpy as np
import pytest
import torch

import oracle
import paper_2208_04187_amd as pkg
from synthetic_inputs import codec_seed, config, draw, draw_config
from tests.parity import check_against_oracle, gpu_roundtrip, to_host_array

pytestmark = pytest.mark.gpu


def _relu_normal(shape, seed, dtype=torch.float32):
    g = torch.Generator().manual_seed(seed)
    return torch.relu(torch.randn(shape, generator=g)).to(dtype)


# ---------------------------------------------------------------- small and medium shapes

TILE_CASES = [
    # shape, B, b                     what it exercises
    ((3, 5, 56, 56), 8, 2),           # 7x7 full blocks, float4 rows, several planes per workgroup
    ((2, 3, 112, 112), 8, 2),         # one plane per workgroup, > 48 KB of LDS
    ((4, 7, 28, 28), 8, 2),           # ragged 8/8/8/4 blocks, padded item slots
    ((5, 9, 14, 14), 8, 2),           # 8+6 blocks, float2 rows
    ((8, 33, 7, 7), 8, 2),            # map smaller than the block: 1x1 LFC, scalar rows, odd plane size
    ((2, 3, 55, 55), 4, 4),           # 13 full blocks + one of 3, odd plane size, 4-bit codes
    ((3, 4, 32, 32), 4, 2),
    ((6, 10, 16, 16), 4, 2),
    ((9, 5, 8, 8), 4, 2),
    ((40, 13, 4, 4), 4, 2),           # one block per plane, one word per plane
    ((2, 16, 32, 32), 8, 4),
    ((1, 1, 190, 190), 8, 2),         # a single large plane in LDS (144 KB)
    ((3, 2, 24, 40), 8, 4),           # H != W
    ((2, 2, 9, 6), 4, 2),             # H*W not a multiple of 4 with even W
    ((1, 3, 5, 3), 8, 2),
    ((1, 1, 1, 1), 4, 2),
    ((300, 7, 7, 7), 8, 4),           # last workgroup holds a partial chunk
    ((3, 5, 56, 56), 8, 4),           # 4-bit codes with a short last round (pair-per-lane tail)
    ((4, 7, 28, 28), 8, 4),
    ((5, 9, 14, 14), 8, 4),
    ((7, 11, 12, 12), 4, 2),
    ((2, 3, 64, 64), 8, 2),           # 16 KB plane
    ((2, 3, 72, 72), 8, 2),           # above the one-wavefront budget: four-wavefront tile kernel
    ((3, 3, 40, 40), 4, 4),
    ((3, 4, 48, 48), 4, 2),           # plane kept in registers, one wavefront, B = 4
    ((2, 3, 50, 44), 8, 2),           # same kernel, ragged blocks both ways, ragged last code word
    ((2, 3, 50, 44), 8, 4),
    ((2, 2, 96, 96), 8, 2),           # plane kept in registers, four wavefronts
    ((1, 3, 100, 92), 8, 4),          # four wavefronts, ragged blocks
    ((9, 1, 56, 56), 8, 2),           # 9 planes: the last workgroup handles one plane only
    ((3, 7, 24, 40), 8, 2),           # chunk of small planes, 15 blocks per plane (not a power of two)
    ((5, 5, 20, 12), 4, 2),           # chunk kernel, 15 blocks, ragged last chunk
    ((2, 3, 22, 18), 8, 4),           # chunk kernel, float2 halves in different blocks, ragged blocks both ways
    ((3, 67, 6, 6), 4, 2),            # chunk kernel, 92 planes per chunk, pad bytes after every plane
    ((1, 2, 44, 44), 4, 4),           # chunk kernel, one plane per chunk, 121 blocks (two rounds of block slots)
]

# 8-bit codes (the Q = 8 column of the paper's bit-width ablation): one shape per kernel family
B8_CASES = [
    ((3, 5, 56, 56), 8, 8), ((2, 2, 96, 96), 8, 8), ((4, 7, 28, 28), 8, 8), ((5, 9, 14, 14), 8, 8),
    ((37, 9, 7, 7), 8, 8), ((2, 3, 72, 72), 8, 8), ((2, 3, 55, 55), 4, 8), ((2, 3, 36, 36), 12, 8),
    ((3, 4, 32, 32), 4, 8), ((2, 2, 9, 6), 4, 8), ((1, 2, 300, 300), 8, 8), ((2, 3, 50, 44), 8, 8),
    ((6, 5, 10, 10), 8, 8),
]

# 1-D maps (Appendix D): Minibatch x Channel x N is the H = 1 case
ONE_D_CASES = [
    ((4, 6, 1, 64), 8, 2), ((3, 5, 1, 197), 8, 2), ((2, 8, 1, 3136), 64, 2), ((7, 3, 1, 128), 16, 4),
    ((5, 4, 1, 50), 64, 2), ((2, 64, 1, 1024), 8, 2), ((2, 3, 1, 2048), 4, 4), ((3, 2, 1, 12544), 8, 2),
]

# enough planes that a workgroup takes several chunks one after the other
MANY_PLANE_CASES = [
    ((2048, 64, 14, 14), 8, 2),
    ((512, 129, 28, 28), 8, 4),
]

ANY_CASES = [
    ((2, 3, 20, 24), 1, 2),           # B = 1: LFC is x itself
    ((2, 3, 20, 24), 2, 4),
    ((2, 3, 20, 24), 3, 2),
    ((2, 3, 36, 36), 12, 2),          # block sizes of the paper's sweep
    ((2, 2, 36, 36), 18, 2),
    ((2, 3, 56, 56), 64, 2),          # block larger than the map
    ((1, 2, 300, 300), 8, 2),         # plane too large for LDS: vector workgroup-per-plane kernel
    ((1, 2, 301, 299), 8, 2),         # same, odd extents: scalar workgroup-per-plane kernel
    ((2, 3, 224, 224), 12, 4),        # image-sized plane, ragged blocks of 8
    ((2, 2, 33, 17), 16, 4),
    ((5, 13, 7, 5), 16, 4),           # one-block planes under a block size the tiled kernels do not cover
    ((70, 3, 7, 7), 64, 2),           # 210 planes: three full rounds of 64 and a ragged one
]


@pytest.mark.parametrize("shape,B,b", MANY_PLANE_CASES)
def test_matches_oracle_many_planes(shape, B, b):
    x = _relu_normal(shape, 2000 + sum(shape))
    st = check_against_oracle(x, B, b, seed=0xABCDEF ^ B, threads=16, require_exact=True)
    assert st["exact"]


@pytest.mark.parametrize("shape,B,seed,gen", [((2048, 512, 4, 4), 4, 123, 5), ((1024, 1024, 5, 6), 3, 77, 6)])
def test_8bit_codes_where_the_scaled_maximum_exceeds_the_top_code(shape, B, seed, gen):
    """With b = 8 the plane maximum scales to 255 plus a few ulp in about one plane in seven, and a
    random term close to 1 then carries the sum to 256: the code must saturate at 255 (six resp. two
    such elements in these inputs; the first shape runs the register kernel, the second the general one)."""
    x = _relu_normal(shape, gen)
    ref, dbg = oracle.compress(x.numpy(), B, 8, seed, threads=16, debug=True)
    s = np.floor(dbg["t"].reshape(-1).astype(np.float64) + dbg["r"].reshape(-1).astype(np.float64) / 65536.0)
    assert (s >= 256).sum() >= 2
    packed = pkg.division_compress(x.to("cuda:0"), B, 8, seed)
    torch.cuda.synchronize()
    assert np.array_equal(packed.cpu().numpy(), ref)


@pytest.mark.parametrize("shape,B,b", TILE_CASES + ANY_CASES + B8_CASES + ONE_D_CASES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_matches_oracle_small(shape, B, b, dtype):
    x = _relu_normal(shape, 1000 + sum(shape) + B + b, dtype)
    st = check_against_oracle(x, B, b, seed=0x1234_5678_9ABC_DEF0 ^ B, require_exact=True)
    assert st["exact"]


def test_unaligned_input_pointer_takes_scalar_loads():
    base = torch.relu(torch.randn(1 + 3 * 5 * 56 * 56, generator=torch.Generator().manual_seed(5)))
    xd = base.to("cuda:0")[1:].view(3, 5, 56, 56)
    assert xd.data_ptr() % 16 == 4
    packed = pkg.division_compress(xd, 8, 2, 77)
    torch.cuda.synchronize()
    ref = oracle.compress(base[1:].view(3, 5, 56, 56).contiguous().numpy(), 8, 2, 77)
    assert np.array_equal(packed.cpu().numpy(), ref)


def test_signed_and_heavy_tailed_values():
    g = torch.Generator().manual_seed(9)
    x = torch.randn((4, 6, 28, 28), generator=g) * torch.exp(3 * torch.randn((4, 6, 1, 1), generator=g))
    x[0, 0] = 0.0                       # an all-zero plane: degenerate range
    x[0, 1] = 3.25                      # a constant plane
    x[1, 2, 5, 5] = 1e30                # one huge outlier
    for b in (2, 4):
        assert check_against_oracle(x, 8, b, seed=3, require_exact=True)["exact"]


# ---------------------------------------------------------------- invariants on the GPU path

def test_B1_roundtrip_is_identity():
    x = torch.randn((2, 3, 12, 20), generator=torch.Generator().manual_seed(2))
    gp, gx = gpu_roundtrip(x, 1, 2, 5)
    s = oracle.split_packed(gp, tuple(x.shape), 1, 2)
    assert np.array_equal(s["lfc"].reshape(x.shape), x.numpy())
    assert not s["codes"].any() and not s["meta"][:, 1].any()
    assert torch.equal(gx, x)


@pytest.mark.parametrize("shape,B", [((3, 4, 56, 56), 8), ((2, 5, 14, 14), 8), ((2, 3, 55, 55), 4)])
def test_block_constant_input_has_zero_hfc(shape, B):
    N, C, H, W = shape
    LH, LW = -(-H // B), -(-W // B)
    g = torch.Generator().manual_seed(4)
    vals = torch.randint(-64, 64, (N, C, LH, LW), generator=g).float() / 8       # exactly summable
    x = vals.repeat_interleave(B, 2).repeat_interleave(B, 3)[:, :, :H, :W].contiguous()
    gp, gx = gpu_roundtrip(x, B, 2, 1)
    s = oracle.split_packed(gp, shape, B, 2)
    assert np.array_equal(s["lfc"].reshape(N, C, LH, LW), vals.numpy())
    assert not s["codes"].any() and not s["meta"][:, 1].any()
    assert torch.equal(gx, x)


def test_error_bound_and_extreme_codes():
    x = _relu_normal((6, 8, 28, 28), 6)
    for b in (2, 4):
        L = (1 << b) - 1
        gp, gx = gpu_roundtrip(x, 8, b, 21)
        s = oracle.split_packed(gp, tuple(x.shape), 8, b)
        Delta = torch.from_numpy(s["meta"][:, 1].copy()).view(6, 8, 1, 1)
        assert torch.all((gx - x).abs() <= Delta * (1 + 1e-5) + 1e-6)
        q = oracle.unpack_codes(s["codes"], 784, b)
        assert np.all(q.min(1) == 0) and np.all(q.max(1) == L)


def test_deterministic_and_independent_of_neighbours():
    x = _relu_normal((16, 16, 14, 14), 8)
    a, _ = gpu_roundtrip(x, 8, 2, 9)
    bb, _ = gpu_roundtrip(x, 8, 2, 9, prefill=0x00)
    assert np.array_equal(a, bb)
    # the first planes of a larger batch compress to the same bytes as on their own:
    # results do not depend on how planes are grouped into workgroups
    sub = x[:3].contiguous()
    c, _ = gpu_roundtrip(sub, 8, 2, 9)
    sa, sc = oracle.split_packed(a, tuple(x.shape), 8, 2), oracle.split_packed(c, tuple(sub.shape), 8, 2)
    for k in ("codes", "meta", "lfc"):
        assert np.array_equal(sa[k][:48], sc[k])


def test_unbiased_over_seeds_on_gpu():
    K = 512
    x = _relu_normal((1, 4, 16, 16), 10)
    xd = x.to("cuda:0")
    acc = torch.zeros_like(xd, dtype=torch.float64)
    for seed in range(K):
        p = pkg.division_compress(xd, 8, 2, seed)
        acc += pkg.division_decompress(p, tuple(x.shape), 8, 2).double()
    mean = (acc / K).cpu()
    s = oracle.split_packed(p.cpu().numpy(), tuple(x.shape), 8, 2)
    Delta = torch.from_numpy(s["meta"][:, 1].copy()).view(1, 4, 1, 1).double()
    err = (mean - x.double()).abs()
    assert torch.all(err <= 4.5 * Delta * 0.5 / K ** 0.5 + 1e-6)
    assert err.mean() < 0.5 * (Delta * 0.5 / K ** 0.5).mean() * 2


def test_runs_on_a_side_stream():
    x = _relu_normal((4, 8, 56, 56), 11).to("cuda:0")
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        p = pkg.division_compress(x, 8, 2, 4, stream=st)
        y = pkg.division_decompress(p, tuple(x.shape), 8, 2, stream=st)
    st.synchronize()
    ref = oracle.compress(x.cpu().numpy(), 8, 2, 4)
    assert np.array_equal(p.cpu().numpy(), ref)
    assert np.array_equal(y.cpu().numpy(), oracle.decompress(ref, tuple(x.shape), 8, 2))


def test_error_codes_on_device_buffers():
    x = torch.zeros((1, 1, 8, 8), device="cuda:0")
    need = pkg.division_packed_bytes(1, 1, 8, 8, 4, 2)
    small = torch.empty(need - 16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(pkg.DivisionError) as e:
        pkg.division_compress(x, 4, 2, 0, packed=small)
    assert e.value.code == 2
    big = torch.empty(need + 16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(pkg.DivisionError) as e:
        pkg.division_compress(x, 4, 2, 0, packed=big[1:])
    assert e.value.code == 3
    with pytest.raises(pkg.DivisionError) as e:
        pkg.division_compress(x, 4, 3, 0)
    assert e.value.code == 1


# ---------------------------------------------------------------- several maps of one shape per launch

BATCH_CASES = [
    # shape, B, b, count                one shape per kernel family; 11 maps = one full launch of 8 + one of 3
    ((3, 5, 56, 56), 8, 2, 11),       # plane in registers
    ((2, 2, 96, 96), 8, 4, 3),        # plane in registers, four wavefronts
    ((4, 7, 28, 28), 8, 2, 11),       # one wavefront per chunk
    ((37, 9, 7, 7), 8, 2, 9),         # one-block planes, two-plane decompress path
    ((2, 3, 72, 72), 8, 2, 2),        # four-wavefront tile
    ((2, 3, 36, 36), 12, 2, 5),       # generic kernels
    ((2, 3, 55, 55), 4, 4, 4),
]


@pytest.mark.parametrize("shape,B,b,count", BATCH_CASES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_batch_matches_oracle_per_tensor(shape, B, b, count, dtype):
    xs = [_relu_normal(shape, 7000 + 13 * i + sum(shape), dtype) for i in range(count)]
    seeds = [(0xC0FFEE << 20) + 0x1_0000_0001 * i for i in range(count)]
    xd = [x.to("cuda:0") for x in xs]
    need = pkg.division_packed_bytes(*shape, B, b, dtype)
    packed = [torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda:0") for _ in xs]
    pkg.division_compress_batch(xd, B, b, seeds, packed=packed)
    outs = pkg.division_decompress_batch(packed, shape, B, b, dtype)
    torch.cuda.synchronize()
    for x, seed, p, y in zip(xs, seeds, packed, outs):
        xh, dt = to_host_array(x)
        ref = oracle.compress(xh, B, b, seed, dt)
        assert np.array_equal(p.cpu().numpy(), ref)
        yh, _ = to_host_array(y.cpu())
        assert np.array_equal(yh, oracle.decompress(ref, shape, B, b, dt))


def test_batch_equals_single_calls_and_empty_batch():
    shape, B, b = (6, 10, 14, 14), 8, 2
    xs = [_relu_normal(shape, 7100 + i).to("cuda:0") for i in range(3)]
    seeds = [5, 6, 7]
    pb = pkg.division_compress_batch(xs, B, b, seeds)
    ps = [pkg.division_compress(x, B, b, s) for x, s in zip(xs, seeds)]
    for u, v in zip(pb, ps):
        assert torch.equal(u, v)
    yb = pkg.division_decompress_batch(pb, shape, B, b)
    for p, y in zip(ps, yb):
        assert torch.equal(y, pkg.division_decompress(p, shape, B, b))
    assert pkg.division_compress_batch([], B, b, []) == []
    assert pkg.division_decompress_batch([], shape, B, b) == []
    # one misaligned member rejects the whole batch before any launch
    need = pkg.division_packed_bytes(*shape, B, b)
    big = torch.empty(need + 16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(pkg.DivisionError) as e:
        pkg.division_compress_batch(xs[:2], B, b, seeds[:2], packed=[pb[0], big[1:]])
    assert e.value.code == 3


def test_batch_with_one_unaligned_input_takes_scalar_loads():
    shape, B, b = (2, 3, 28, 28), 8, 2
    base = torch.zeros(2 * 3 * 28 * 28 + 1, device="cuda:0")
    x0 = _relu_normal(shape, 7200)
    x1 = _relu_normal(shape, 7201)
    base[1:].copy_(x1.flatten())
    xs = [x0.to("cuda:0"), base[1:].view(shape)]
    assert xs[1].data_ptr() % 16 == 4
    pb = pkg.division_compress_batch(xs, B, b, [1, 2])
    torch.cuda.synchronize()
    assert np.array_equal(pb[0].cpu().numpy(), oracle.compress(x0.numpy(), B, b, 1))
    assert np.array_equal(pb[1].cpu().numpy(), oracle.compress(x1.numpy(), B, b, 2))


# ---------------------------------------------------------------- the benchmark configurations

def test_config0_small_tensor_exact():
    for k, spec, x in draw_config(0):
        st = check_against_oracle(x, spec.B, spec.b, codec_seed(0, k), require_exact=True)
        assert st["exact"]


@pytest.mark.parametrize("idx", [1, 2, 4])
def test_full_size_fp32_configs(idx):
    total = flips = 0
    for k, spec, x in draw_config(idx):
        st = check_against_oracle(x, spec.B, spec.b, codec_seed(idx, k), threads=16)
        total += st["elements"]
        flips += st["flips"]
        print(f"config {idx} tensor {k} {spec.name}: exact={st['exact']} flips={st['flips']}", flush=True)
    assert flips <= 1e-6 * total


@pytest.mark.parametrize("idx", [1, 2])
def test_full_size_configs_in_batch_launches(idx):
    """The launch configuration the benchmark times: consecutive maps of one shape share a launch."""
    drawn = list(draw_config(idx))
    groups = []
    for k, spec, x in drawn:
        key = (tuple(x.shape), spec.B, spec.b)
        if groups and groups[-1][0] == key and len(groups[-1][1]) < 8:
            groups[-1][1].append((k, x))
        else:
            groups.append((key, [(k, x)]))
    for (shape, B, b), members in groups:
        xs = [x.to("cuda:0") for _, x in members]
        seeds = [codec_seed(idx, k) for k, _ in members]
        need = pkg.division_packed_bytes(*shape, B, b)
        packed = [torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda:0") for _ in xs]
        pkg.division_compress_batch(xs, B, b, seeds, packed=packed)
        outs = pkg.division_decompress_batch(packed, shape, B, b)
        torch.cuda.synchronize()
        for (k, x), seed, pk, y in zip(members, seeds, packed, outs):
            ref = oracle.compress(x.numpy(), B, b, seed, threads=16)
            assert np.array_equal(pk.cpu().numpy(), ref), f"config {idx} tensor {k}"
            assert np.array_equal(y.cpu().numpy(), oracle.decompress(ref, shape, B, b, threads=16)), f"config {idx} tensor {k}"
        del xs, packed, outs
        torch.cuda.empty_cache()



def test_full_size_bf16_config3():
    for k, spec, x in draw_config(3):
        xb = x.to(torch.bfloat16)
        del x
        st = check_against_oracle(xb, spec.B, spec.b, codec_seed(3, k), threads=16)
        print(f"config 3 {spec.name}: exact={st['exact']} flips={st['flips']}", flush=True)
        assert st["flips"] <= 1e-6 * st["elements"]


# ---------------------------------------------------------------- block means at binary32 rounding midpoints

def _midpoint_plane(rng, cnt_side=7):
    """A cnt_side x cnt_side plane (one block when B=8) whose exact mean is a binary32
    rounding midpoint, plus neighbours a hair above and below it."""
    from fractions import Fraction
    n = cnt_side * cnt_side
    k = int(rng.integers(1 << 23, 1 << 24))
    M = Fraction(2 * k + 1, 1 << 26)                      # odd multiple of 2^-26 in [0.25, 0.5): a midpoint
    vals = [Fraction(int(v), 1 << 25) for v in rng.integers(1 << 23, 1 << 24, n - 3)]
    R = n * M - sum(vals)
    u = Fraction(float(np.float32(float(R / 2))))
    w = Fraction(float(np.float32(float(R - u))))
    t = R - u - w
    assert Fraction(float(np.float32(float(t)))) == t    # the remainder is itself a binary32 value
    planes = []
    for eps in (Fraction(0), Fraction(1, 1 << 44), -Fraction(1, 1 << 44)):
        tt = t + eps
        if Fraction(float(np.float32(float(tt)))) != tt:
            continue
        p = np.array([float(v) for v in vals] + [float(u), float(w), float(tt)], np.float32)
        assert sum(Fraction(float(v)) for v in p) == n * M + eps
        planes.append(rng.permutation(p).reshape(cnt_side, cnt_side))
    return planes


def test_block_mean_on_rounding_midpoints():
    rng = np.random.default_rng(77)
    planes = []
    while len(planes) < 96:
        planes += _midpoint_plane(rng)
    x = torch.from_numpy(np.stack(planes[:96]).reshape(4, 24, 7, 7))
    st = check_against_oracle(x, 8, 2, seed=5, require_exact=True)
    assert st["exact"]


@pytest.mark.parametrize("shape", [(2, 3, 112, 112), (3, 5, 56, 56), (5, 7, 28, 28), (9, 7, 14, 14), (11, 13, 7, 7),
                                   (2, 3, 24, 40), (2, 2, 55, 55), (2, 3, 64, 64), (1, 2, 224, 224)])
def test_codes_on_exact_ties_of_the_stochastic_rounding(shape):
    # maps built so that t + u is exactly an integer, one step of u below it or 2^-25 below it for the random
    # bits the element really gets (tests/test_oracle_rounding_pins.py derives the expected codes by hand)
    from tests.test_oracle_rounding_pins import tie_map
    seed = 0xBEEF
    xh, expect = tie_map(shape, seed)
    x = torch.from_numpy(xh)
    st = check_against_oracle(x, 8, 2, seed=seed, require_exact=True)
    assert st["exact"]
    gp, _ = gpu_roundtrip(x, 8, 2, seed)
    s = oracle.split_packed(gp, shape, 8, 2, oracle.F32)
    q = oracle.unpack_codes(s["codes"], shape[2] * shape[3], 2)
    for pl, e in enumerate(expect):
        for i, c in e.items():
            assert int(q[pl, i]) == c, (pl, i)


def test_bfloat16_map_is_rebuilt_with_round_to_nearest_even():
    # hand-made packed buffers: H^L = 1, delta = 0, Delta = 2^-9, 8-bit codes 0..255 over 56 x 56 elements, so that
    # xhat = 1 + code * 2^-9 lands on, just below and just above halfway between neighbouring bfloat16 values
    shape, B, b = (2, 3, 56, 56), 64, 8
    p = np.zeros(oracle.packed_bytes(*shape, B, b, oracle.BF16), dtype=np.uint8)
    s = oracle.split_packed(p, shape, B, b, oracle.BF16)
    codes = (np.arange(56 * 56, dtype=np.uint32) * 7 + 3) % 256
    s["codes"][:] = (codes.reshape(-1, 4) << (8 * np.arange(4, dtype=np.uint32))).sum(1).astype(np.uint32)[None, :]
    s["meta"][:, 0] = 0.0
    s["meta"][:, 1] = 2.0 ** -9
    s["lfc"][:] = 0x3F80
    want = torch.tensor(1.0 + codes.astype(np.float64) * 2.0 ** -9, dtype=torch.float32).to(torch.bfloat16)
    y = pkg.division_decompress(torch.from_numpy(p).to("cuda:0"), shape, B, b, torch.bfloat16)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().view(torch.int16).numpy().reshape(6, -1), oracle.decompress(p, shape, B, b, oracle.BF16).view(np.int16).reshape(6, -1))
    for pl in range(6):
        assert torch.equal(y.cpu().view(torch.int16).reshape(6, -1)[pl], want.view(torch.int16))


# 1-bit codes (Q = 1): the register, strip, lane, items and units kernels on the shapes they take, the general kernel elsewhere
ONE_BIT_CASES = [
    # shape, B, compress kernel, decompress kernel (of fp32 maps)
    ((3, 5, 56, 56), 8, "compress_regs<float, 1, 8, 1>", "decompress_stream"),
    ((3, 5, 56, 56), 4, "compress_regs<float, 1, 4, 1>", "decompress_stream"),
    ((3, 5, 56, 56), 12, "compress_regs<float, 1, 0, 1>", "decompress_stream"),
    ((2, 3, 48, 48), 8, "compress_regs<float, 1, 8, 1>", "decompress_stream"),      # rounds past the plane
    ((2, 3, 47, 44), 8, "compress_regs<float, 1, 8, 1>", "decompress_stream"),      # 517 units: the last byte holds one unit
    ((2, 3, 51, 60), 4, "compress_regs<float, 1, 4, 1>", "decompress_stream"),      # 765 units
    ((2, 3, 112, 112), 8, "compress_regs<float, 1, 8, 4>", "decompress_stream"),
    ((2, 3, 96, 96), 8, "compress_regs<float, 1, 8, 4>", "decompress_stream"),
    ((1, 3, 97, 92), 8, "compress_regs<float, 1, 8, 4>", "decompress_stream"),      # 2231 units
    ((1, 2, 224, 224), 8, "compress_regs<float, 1, 8, 16>", "decompress_stream"),
    ((2, 3, 160, 160), 8, "compress_regs<float, 1, 8, 16>", "decompress_stream"),
    ((2, 3, 1, 3136), 8, "compress_regs<float, 1, 8, 1>", "decompress_stream"),
    ((2, 3, 28, 28), 8, "compress_strip<float, 1, 28, 8>", "decompress_stream"),
    ((1, 5, 28, 28), 8, "compress_strip<float, 1, 28, 8>", "decompress_stream"),    # a ragged last round
    ((2, 3, 20, 28), 8, "compress_strip<float, 1, 28, 8>", "decompress_stream"),
    ((2, 3, 27, 28), 8, "compress_strip<float, 1, 28, 8>", "decompress_stream"),    # 756 bits: strips end inside a word
    ((2, 3, 28, 28), 12, "compress_strip<float, 1, 28, 12>", "decompress_stream"),
    ((2, 3, 28, 28), 18, "compress_strip<float, 1, 28, 18>", "decompress_table"),
    ((4, 6, 14, 14), 8, "compress_strip<float, 1, 14, 8>", "decompress_table"),
    ((1, 7, 14, 14), 8, "compress_strip<float, 1, 14, 8>", "decompress_table"),
    ((2, 3, 10, 14), 8, "compress_strip<float, 1, 14, 8>", "decompress_table"),
    ((2, 5, 14, 14), 12, "compress_strip<float, 1, 14, 12>", "decompress_table"),
    ((3, 5, 32, 32), 4, "compress_strip<float, 1, 32, 4>", "decompress_stream"),
    ((1, 1, 32, 32), 8, "compress_strip<float, 1, 32, 8>", "decompress_stream"),
    ((2, 3, 32, 32), 16, "compress_strip<float, 1, 32, 16>", "decompress_stream"),
    ((3, 5, 16, 16), 8, "compress_strip<float, 1, 16, 8>", "decompress_stream"),
    ((3, 5, 16, 16), 4, "compress_strip<float, 1, 16, 4>", "decompress_stream"),
    ((2, 5, 16, 16), 12, "compress_strip<float, 1, 16, 12>", "decompress_stream"),
    ((5, 7, 7, 7), 8, "compress_lane<float, 1>", "decompress_lane"),
    ((3, 67, 7, 7), 8, "compress_lane<float, 1>", "decompress_lane"),
    ((2, 3, 5, 5), 8, "compress_lane<float, 1>", "decompress_lane"),
    ((1, 1, 1, 1), 8, "compress_lane<float, 1>", "decompress_lane"),
    ((2, 9, 1, 96), 64, "compress_line<float, 1, 12, 6>", "decompress_stream"),
    ((2, 9, 1, 768), 8, "compress_line<float, 1, 6, 1>", "decompress_stream"),
    ((2, 9, 1, 768), 64, "compress_line<float, 1, 6, 1>", "decompress_stream"),
    ((5, 9, 1, 196), 16, "compress_line<float, 1, 4, 1>", "decompress_stream"),      # 49 vectors: the last byte holds one
    ((3, 7, 1, 100), 8, "compress_line<float, 1, 4, 1>", "decompress_stream"),       # 25 vectors
    ((7, 9, 1, 24), 8, "compress_line<float, 1, 12, 12>", "decompress_stream"),
    ((2, 3, 1, 3072), 64, "compress_regs<float, 1, 0, 1>", "decompress_stream"),
    ((2, 3, 1, 3072), 4096, "compress_one<float, 1, 13>", "decompress_stream"),
    ((3, 5, 56, 56), 64, "compress_one<float, 1, 13>", "decompress_stream"),
    ((3, 5, 28, 28), 64, "compress_one<float, 1, 13>", "decompress_stream"),
    ((3, 67, 14, 14), 64, "compress_one<float, 1, 13>", "decompress_"),               # 49 vectors per plane
    ((3, 5, 6, 6), 8, "compress_items<float, 1, 8, 2, 8>", "decompress_"),
    ((3, 5, 12, 12), 64, "compress_one<float, 1, ", "decompress_"),                   # 36 vectors
    ((3, 5, 6, 10), 32, "compress_one<float, 1, ", "decompress_"),                    # 15 vectors
    ((3, 5, 54, 57), 64, "compress_units<float, 1, 2>", "decompress_"),
    ((2, 3, 64, 64), 8, "compress_tile<float, 1, 8, 4, 256>", "decompress_stream"),
    ((2, 3, 40, 40), 4, "compress_tile<float, 1, 4, 4, 256>", "decompress_stream"),
    ((2, 3, 20, 30), 4, "compress_tile<float, 1, 4, 2, 256>", "decompress_"),
    ((5, 7, 11, 15), 4, "compress_rowstrip<float, 1, 15, 4>", "decompress_stream_any"),
    ((5, 7, 15, 11), 4, "compress_tile<float, 1, 4, 1, 256>", "decompress_stream_any"),
    ((2, 3, 44, 46), 8, "compress_tile<float, 1, 8, 2, 256>", "decompress_"),
    ((1, 2, 300, 300), 8, "compress_any<float, 1>", "decompress_"),
    ((2, 3, 28, 28), 3, "compress_any<float, 1>", "decompress_table"),
    ((2, 2, 100, 37), 8, "compress_units<float, 1, 2>", "decompress_table"),
    ((2, 3, 53, 53), 4, "compress_units<float, 1, 2>", "decompress_stream_any"),
    ((2, 3, 57, 57), 8, "compress_units<float, 1, 2>", "decompress_stream_any"),
    ((2, 3, 55, 55), 8, "compress_rowstrip<float, 1, 55, 8>", "decompress_stream_any"),
    ((3, 2, 33, 17), 12, "compress_units<float, 1, 1>", "decompress_stream_any"),
    ((2, 3, 29, 29), 8, "compress_units<float, 1, 1>", "decompress_stream_any"),       # 841 elements: a lone unit in the last byte
    ((2, 3, 37, 37), 8, "compress_units<float, 1, 1>", "decompress_stream_any"),
    ((2, 3, 73, 73), 8, "compress_units<float, 1, 4>", "decompress_stream_any"),
    ((1, 3, 125, 125), 8, "compress_units<float, 1, 8>", "decompress_stream_any"),
    ((1, 2, 147, 147), 8, "compress_tile<float, 1, 8, 1, 256>", "decompress_stream_any"),   # sixteen wavefronts per plane: no 1-bit instance of the units kernel
    ((1, 2, 147, 147), 18, "compress_any<float, 1>", "decompress_stream_any"),
    ((5, 7, 19, 19), 8, "compress_units<float, 1, 0>", "decompress_stream_any"),        # 16 lanes per plane
    ((5, 7, 18, 19), 4, "compress_units<float, 1, 0>", "decompress_stream_any"),
    ((5, 7, 11, 11), 8, "compress_tile<float, 1, 8, 1, 256>", "decompress_stream_any"),
    ((3, 5, 9, 6), 4, "compress_items<float, 1, 4, 2, 4>", "decompress_"),
    ((4, 8, 8, 8), 4, "compress_items<float, 1, 4, 4, 4>", "decompress_stream"),
    ((4, 8, 8, 8), 8, "compress_items<float, 1, 8, 4, 8>", "decompress_stream"),
    ((9, 8, 4, 4), 4, "compress_items<float, 1, 4, 4, 4>", "decompress_stream"),
    ((3, 8, 12, 20), 8, "compress_items", "decompress_stream"),
]


@pytest.mark.parametrize("shape,B,ckern,dkern", ONE_BIT_CASES)
@pytest.mark.parametrize("mode", ["f32", "bf16", "c16"])
def test_one_bit_codes_match_oracle(shape, B, ckern, dkern, mode):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    c16 = mode == "c16"
    tn = {"f32": "float", "bf16": "bf16_t", "c16": "f32c16_t"}[mode]
    if mode != "bf16":     # (2-byte elements: other vector counts, so sometimes another kernel)
        assert pkg.division_kernel_name(0, shape, B, 1, dtype, c16=c16).startswith(ckern.replace("float", tn))
    if mode == "f32":
        assert pkg.division_kernel_name(1, shape, B, 1, dtype).startswith(dkern)
    _check_variant(shape, B, 1, mode)
    # pad bits and bytes of a buffer that held something else before
    dt = oracle.F32_C16 if c16 else (oracle.BF16 if mode == "bf16" else oracle.F32)
    x = _relu_normal(shape, 5 + B, dtype)
    xh, _ = to_host_array(x)
    pk = torch.full((pkg.division_packed_bytes(*shape, B, 1, dtype, c16),), 0xFF, dtype=torch.uint8, device="cuda:0")
    pkg.division_compress(x.to("cuda:0"), B, 1, 99, packed=pk, c16=c16)
    torch.cuda.synchronize()
    assert np.array_equal(pk.cpu().numpy(), oracle.compress(xh, B, 1, 99, dt, threads=16))
    # and the ratio the codec was asked for: one bit per element + H^L + scale
    n = shape[0] * shape[1] * shape[2] * shape[3]
    if shape[2] * shape[3] >= 256:
        assert pkg.division_packed_bytes(*shape, B, 1, dtype, c16) < n * (2 if mode == "bf16" else 4) / 4


# block sizes and ragged edges that give blocks of 98, 196, 198 or 150 elements: counts whose binary64 reciprocal, times the
# sum, lands beside an exact tie instead of on it
@pytest.mark.parametrize("shape,B", [((4, 6, 56, 56), 14), ((4, 6, 28, 28), 14), ((4, 6, 14, 14), 16), ((4, 6, 14, 14), 64),
                                      ((4, 6, 47, 76), 18), ((4, 6, 29, 36), 18), ((4, 6, 7, 14), 16), ((1, 12, 300, 300), 14),
                                      ((2, 6, 150, 150), 14), ((4, 6, 35, 35), 14), ((4, 6, 17, 17), 14), ((4, 6, 1, 770), 98),
                                      ((4, 6, 1, 708), 256), ((4, 6, 170, 170), 15), ((8, 6, 13, 14), 6), ((2, 6, 250, 250), 14),
                                      ((4, 6, 56, 56), 12), ((4, 6, 35, 35), 3), ((2, 6, 203, 200), 28),
                                      ((2, 6, 7, 7, 4), 8), ((2, 6, 2, 7, 7), 8), ((2, 6, 7, 28, 28), 28), ((1, 12, 14, 30, 34), 14)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_block_mean_that_is_a_subnormal_number(shape, B, dtype):
    # integers times the smallest subnormal: a block mean is sum / count in units of 2^-149 (2^-133 for bfloat16), so
    # binary32 rounds it to an integer, and with an even count that is no power of two many means are exact ties
    g = torch.Generator().manual_seed(sum(shape) + B)
    unit = 2.0 ** -149 if dtype == torch.float32 else 2.0 ** -133
    top = 3000 if dtype == torch.float32 else 100
    x = (torch.randint(-top, top, shape, generator=g).double() * unit).float().to(dtype)
    xh, dt = to_host_array(x)
    ref = oracle.compress(xh, B, 2, 5, dt, threads=16)
    lfc = oracle.split_packed(ref, shape, B, 2, dt)["lfc"]
    lf = (oracle.bf16_to_f32(lfc) if dtype == torch.bfloat16 else lfc).astype(np.float64)
    assert np.abs(lf).max() < 2.0 ** -126 and np.count_nonzero(lf) > lf.size // 2          # the means are subnormal
    three = len(shape) == 5
    pk = (pkg.division_compress_3d if three else pkg.division_compress)(x.to("cuda:0"), B, 2, 5)
    torch.cuda.synchronize()
    got = oracle.split_packed(pk.cpu().numpy(), shape, B, 2, dt)["lfc"]
    assert np.array_equal(got.view(np.uint8), lfc.view(np.uint8)), \
        (pkg.division_kernel_name_3d if three else pkg.division_kernel_name)(0, shape, B, 2, dtype)
    assert np.array_equal(pk.cpu().numpy(), ref)


def test_descriptor_array_calls_serve_a_mixed_step():
    """Maps of different shapes, dimensionalities, types and parameters in one call each way; every map
    must come out exactly as its single-map call gives it (and as the oracle does)."""
    g = torch.Generator().manual_seed(4242)
    specs = [((2, 8, 56, 56), 8, 2, torch.float32), ((2, 16, 28, 28), 8, 2, torch.float32), ((2, 8, 56, 56), 8, 2, torch.float32),
             ((3, 5, 14, 14), 8, 4, torch.bfloat16), ((2, 3, 4, 12, 12), 4, 2, torch.float32), ((2, 16, 28, 28), 8, 2, torch.float32),
             ((4, 6, 1, 768), 8, 4, torch.float32), ((2, 8, 56, 56), 12, 2, torch.float32), ((2, 9, 7, 7), 8, 2, torch.float32),
             ((2, 16, 28, 28), 8, 2, torch.float32)] + [((2, 8, 56, 56), 8, 2, torch.float32)] * 9     # 11 maps of one shape: two launches
    xs = [torch.relu(torch.randn(sh, generator=g)).to(dt).to("cuda:0") for sh, _, _, dt in specs]
    Bs, bs = [s[1] for s in specs], [s[2] for s in specs]
    seeds = [1000 + 7 * i for i in range(len(specs))]
    pks = pkg.division_compress_maps(xs, Bs, bs, seeds)
    ys = pkg.division_decompress_maps(pks, [s[0] for s in specs], Bs, bs, [s[3] for s in specs])
    torch.cuda.synchronize()
    for i, (sh, B, b, dt) in enumerate(specs):
        xh, odt = to_host_array(xs[i].cpu())
        ref = oracle.compress(xh, B, b, seeds[i], odt)
        assert np.array_equal(pks[i].cpu().numpy(), ref), (i, sh)
        yh, _ = to_host_array(ys[i].cpu())
        assert np.array_equal(yh, oracle.decompress(ref, sh, B, b, odt)), (i, sh)
    assert pkg.division_compress_maps([], 8, 2, []) == []
    with pytest.raises(pkg.DivisionError):
        pkg.division_compress_maps(xs[:2], [8, 8], [2, 3], [1, 2])


# ---------------------------------------------------------------- HIP graph capture

def test_compress_and_decompress_replay_from_a_hip_graph():
    """The library allocates nothing and records no memset, so a step can be captured once and
    replayed; every replay (with the program's own eager work in between) must reproduce the eager result."""
    shapes = [((6, 8, 56, 56), 8, 2), ((5, 9, 14, 14), 8, 2), ((37, 9, 7, 7), 8, 2), ((4, 7, 28, 28), 8, 4)]
    xs = [torch.empty(s, device="cuda:0") for s, _, _ in shapes]
    packed = [torch.empty(pkg.division_packed_bytes(*s, B, b), dtype=torch.uint8, device="cuda:0") for s, B, b in shapes]
    outs = [torch.empty(s, device="cuda:0") for s, _, _ in shapes]

    def step(stream=None):
        for x, pk, y, (s, B, b) in zip(xs, packed, outs, shapes):
            pkg.division_compress(x, B, b, 1234, packed=pk, stream=stream)
            pkg.division_decompress(pk, s, B, b, out=y, stream=stream)

    def fill(k):
        for i, (x, (s, _, _)) in enumerate(zip(xs, shapes)):
            x.copy_(_relu_normal(s, 9000 + 10 * k + i))

    fill(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(side)                      # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(side)
    for k in range(1, 4):
        fill(k)                         # eager work between replays
        for pk in packed:
            pk.fill_(0xEE)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [(pk.clone(), y.clone()) for pk, y in zip(packed, outs)]
        for pk in packed:
            pk.fill_(0x11)
        step()                          # the same step, eagerly
        torch.cuda.synchronize()
        for (gp, gy), pk, y, x, (s, B, b) in zip(got, packed, outs, xs, shapes):
            assert torch.equal(gp, pk) and torch.equal(gy, y)
            assert np.array_equal(gp.cpu().numpy(), oracle.compress(x.cpu().numpy(), B, b, 1234))


# ---------------------------------------------------------------- seeded sweep over shapes and parameters

def _sweep_cases(n, seed):
    rng = np.random.default_rng(seed)
    sizes = [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 13, 14, 16, 17, 20, 24, 28, 31, 32, 33, 40, 48, 55, 56, 57, 64, 72]
    cases = []
    for _ in range(n):
        H, W = int(rng.choice(sizes)), int(rng.choice(sizes))
        if rng.random() < 0.5:
            W = H                                              # square maps are the common case
        B = int(rng.choice([1, 2, 3, 4, 4, 4, 5, 6, 7, 8, 8, 8, 8, 9, 12, 16, 64]))
        b = int(rng.choice([2, 2, 4, 8]))
        N, C = int(rng.integers(1, 6)), int(rng.integers(1, 12))
        if H * W <= 64 and rng.random() < 0.5:
            N, C = int(rng.integers(20, 90)), int(rng.integers(3, 9))      # several rounds of small planes
        cases.append(((N, C, H, W), B, b, bool(rng.random() < 0.3), int(rng.integers(0, 2 ** 63))))
    return cases


@pytest.mark.parametrize("chunk", range(6))
def test_seeded_sweep_of_shapes_block_sizes_and_code_widths(chunk):
    """240 pseudo-random (shape, B, b, dtype, seed) combinations, 40 per test: every kernel family
    and most of their ragged paths; single and batched calls must both be bit-exact."""
    for shape, B, b, bf16, seed in _sweep_cases(240, 20240511)[40 * chunk:40 * (chunk + 1)]:
        dtype = torch.bfloat16 if bf16 else torch.float32
        x = _relu_normal(shape, seed % 100003, dtype)
        xh, dt = to_host_array(x)
        ref = oracle.compress(xh, B, b, seed, dt)
        xd = x.to("cuda:0")
        need = pkg.division_packed_bytes(*shape, B, b, dtype)
        pk = torch.full((need,), 0xA5, dtype=torch.uint8, device="cuda:0")
        pkg.division_compress(xd, B, b, seed, packed=pk)
        pks = pkg.division_compress_batch([xd, xd], B, b, [seed + 1, seed])
        y = pkg.division_decompress(pk, shape, B, b, dtype)
        torch.cuda.synchronize()
        tag = f"shape={shape} B={B} b={b} dtype={dtype} seed={seed}"
        assert np.array_equal(pk.cpu().numpy(), ref), tag
        assert torch.equal(pks[1], pk), tag
        yh, _ = to_host_array(y.cpu())
        assert np.array_equal(yh, oracle.decompress(ref, shape, B, b, dt)), tag


def _sweep_cases_whole_vectors(n, seed0):
    """Maps whose rows are whole 4- or 8-element vectors, under every block size: the register and
    one-block kernels and the vector paths of the general ones."""
    rng = np.random.default_rng(seed0)
    cases = []
    for _ in range(n):
        W = 4 * int(rng.integers(1, 33))
        H = int(rng.choice([1, W, int(rng.integers(1, 130))]))
        B = int(rng.choice([4, 8, 12, 12, 16, 16, 18, 20, 24, 32, 64, 64, 128]))
        b = int(rng.choice([2, 2, 4, 8]))
        N, C = int(rng.integers(1, 5)), int(rng.integers(1, 10))
        if H * W <= 1024 and rng.random() < 0.5:
            N, C = int(rng.integers(8, 40)), int(rng.integers(3, 12))
        mode = str(rng.choice(["f32", "f32", "bf16", "c16"]))
        cases.append(((N, C, H, W), B, b, mode, int(rng.integers(0, 2 ** 63))))
    return cases


@pytest.mark.parametrize("chunk", range(4))
def test_seeded_sweep_of_vector_row_maps_under_every_block_size(chunk):
    for shape, B, b, mode, seed in _sweep_cases_whole_vectors(160, 20260118)[40 * chunk:40 * (chunk + 1)]:
        dtype = torch.bfloat16 if mode == "bf16" else torch.float32
        c16 = mode == "c16"
        dt = oracle.F32_C16 if c16 else (oracle.BF16 if mode == "bf16" else oracle.F32)
        g = torch.Generator().manual_seed(seed % 100003)
        x = (torch.randn(shape, generator=g) * 1.7 - 0.2).to(dtype)
        xh, _ = to_host_array(x)
        ref = oracle.compress(xh, B, b, seed, dt)
        need = pkg.division_packed_bytes(*shape, B, b, dtype, c16)
        pk = torch.full((need,), 0xC3, dtype=torch.uint8, device="cuda:0")
        pkg.division_compress(x.to("cuda:0"), B, b, seed, packed=pk, c16=c16)
        y = pkg.division_decompress(pk, shape, B, b, dtype, c16=c16)
        torch.cuda.synchronize()
        tag = f"shape={shape} B={B} b={b} mode={mode} seed={seed} kernel={pkg.division_kernel_name(0, shape, B, b, dtype, c16=c16)}"
        assert np.array_equal(pk.cpu().numpy(), ref), tag
        yh, _ = to_host_array(y.cpu())
        assert np.array_equal(yh, oracle.decompress(ref, shape, B, b, dt)), tag


# ---------------------------------------------------------------- the block sizes of the paper's sweep (Sec. 5, B ablation)

ROWS_CASES = [
    # shape, B, b                       what it exercises in the general-block-size kernel
    ((8, 24, 56, 56), 12, 2),           # 4 full blocks + one of 8 per side, several planes per chunk, many chunks
    ((8, 24, 56, 56), 16, 2),           # 3 full blocks + one of 8
    ((8, 24, 56, 56), 18, 4),           # 3 full blocks + one of 2
    ((8, 24, 54, 57), 64, 2),           # block larger than the map on a plane that is not whole vectors
    ((7, 19, 28, 28), 12, 2),           # odd plane count: ragged last chunk
    ((7, 19, 28, 28), 18, 8),
    ((5, 33, 14, 14), 12, 4),           # blocks of 12 and 2
    ((3, 5, 112, 112), 16, 2),          # one plane per chunk, 49 blocks
    ((3, 5, 112, 112), 64, 2),          # blocks of 64 and 48
    ((2, 3, 150, 150), 18, 2),          # 90 KB plane, 81 blocks, ragged blocks of 6
    ((6, 11, 7, 100), 16, 2),           # block taller than the map, seven columns of blocks
    ((6, 11, 100, 7), 16, 4),           # block wider than the map
    ((4, 9, 27, 35), 5, 2),             # odd everything: H*W odd, blocks of 5 and 2 / 5 exactly
    ((4, 9, 27, 35), 7, 4),
    ((3, 7, 30, 30), 6, 2),
    ((16, 48, 1, 196), 16, 2),          # 1-D maps
    ((5, 7, 1, 1000), 12, 4),
    ((2, 3, 33, 31), 2, 2),             # tiny blocks: 272 blocks per plane
    ((2, 3, 40, 40), 1, 4),             # B = 1
    ((6, 10, 12, 20), 12, 2),           # planes below 256 elements stay with this kernel: whole-vector rows,
    ((5, 8, 15, 15), 6, 4),             # odd rows,
    ((9, 4, 7, 33), 18, 8),             # wide and flat
]


# planes that are one block (B at least every extent): the flat one-block kernel
ONE_BLOCK_CASES = [
    ((8, 24, 56, 56), 64, 2),           # 784 vectors: all 64 lanes, 13 vectors each (the Swin-T setting B = 64)
    ((7, 19, 28, 28), 64, 4),           # 196 vectors: 16 lanes per plane, 4 planes per wavefront, ragged last wavefront
    ((5, 33, 14, 14), 64, 2),           # 49 vectors: 4 lanes per plane
    ((3, 5, 6, 10), 16, 8),             # 15 vectors
    ((130, 3, 12, 12), 16, 2),          # 390 planes of 36 vectors
    ((8, 8, 1, 3072), 4096, 2),         # 1-D map under one block
    ((9, 7, 1, 52), 64, 4),             # 13 vectors: a lane per plane, 63 planes: one wavefront, one lane idle
    ((2, 3, 56, 56), 128, 8),
    ((3, 3, 10, 16), 18, 2),            # ragged last code word (160 elements at 16 per word: exact) and B = 18
    ((3, 3, 10, 14), 18, 2),            # 140 elements: the last word of a plane is partly pad
]


@pytest.mark.parametrize("shape,B,b", ONE_BLOCK_CASES)
@pytest.mark.parametrize("mode", ["f32", "bf16", "c16"])
def test_one_block_kernel_matches_oracle(shape, B, b, mode):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    c16 = mode == "c16"
    hw = shape[2] * shape[3]
    if mode != "bf16" or hw % 8 == 0:
        assert pkg.division_kernel_name(0, shape, B, b, dtype, c16=c16).startswith("compress_one<")
    _check_variant(shape, B, b, mode)


# 1-D maps (Appendix D; the maps of linear and transformer layers): the register kernel for one row
LINE_CASES = [
    ((32, 16, 1, 768), 8, 4),           # hidden size 768, the B = 8 / Q = 4 setting of the paper's language-model run
    ((6, 50, 1, 96), 64, 2),            # two blocks of 64 and 32 elements
    ((6, 50, 1, 96), 8, 2),
    ((100, 1, 1, 128), 16, 2),          # 128 features, the B = 16 setting of the paper's MLP run
    ((9, 7, 1, 196), 16, 8),            # 49 vectors, short last block
    ((3, 4, 1, 1664), 32, 2),           # 416 vectors: 32 lanes x 13
    ((5, 3, 1, 200), 8, 2),             # 50 vectors
    ((70, 3, 1, 24), 4, 4),             # tiny planes: 6 vectors, 8 lanes per plane, ragged last wavefront
    ((4, 4, 1, 1024), 64, 4),
    # token vectors of a Swin-T under its B = 64: 96 / 192 wide (two / three rounds, several plane groups per
    # wavefront, 9408 planes: XCD-aware order and its tail), 384 / 768 wide (six rounds)
    ((3, 3136, 1, 96), 64, 2),
    ((5, 157, 1, 192), 64, 4),
    ((7, 13, 1, 384), 64, 2),
    ((5, 49, 1, 768), 64, 8),
    ((3, 7, 1, 1536), 64, 2),
]


@pytest.mark.parametrize("shape,B,b", LINE_CASES)
@pytest.mark.parametrize("mode", ["f32", "bf16", "c16"])
def test_one_row_kernel_matches_oracle(shape, B, b, mode):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    if mode != "bf16" or (shape[3] % 8 == 0 and B % 8 == 0):
        assert pkg.division_kernel_name(0, shape, B, b, dtype, c16=mode == "c16").startswith("compress_line<")
    _check_variant(shape, B, b, mode)


# planes of width 28 and 14 under B = 8: the strip kernel (a lane per 28 consecutive elements)
STRIP_CASES = [
    ((3, 171, 28, 28), 2),              # 513 planes: an odd number, the last round holds one plane
    ((2, 64, 28, 28), 4),
    ((1, 33, 28, 28), 8),
    ((5, 41, 14, 14), 2),               # 205 planes in rounds of 8: the last round holds 5
    ((2, 100, 14, 14), 4),
    ((1, 19, 14, 14), 8),
    ((3, 67, 20, 28), 2),               # ragged last block row (4 of 8 rows), lanes 20..31 of a plane idle
    ((3, 67, 32, 28), 4),               # every lane slot in use
    ((3, 67, 3, 28), 2),                # three lanes per plane
    ((3, 67, 9, 28), 8),
    ((3, 67, 16, 14), 2),               # every lane slot in use (8 row pairs)
    ((3, 67, 2, 14), 4),                # one row pair per plane
    ((3, 67, 10, 14), 2),               # ragged last block row (2 of 8 rows)
    ((1, 1, 28, 28), 2), ((1, 1, 14, 14), 2),
    ((9, 600, 14, 14), 2),              # 5400 planes: more than one run of the XCD-aware order and its plain tail
]


@pytest.mark.parametrize("shape,b", STRIP_CASES)
@pytest.mark.parametrize("mode", ["f32", "bf16", "c16"])
def test_strip_kernel_matches_oracle(shape, b, mode):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    assert pkg.division_kernel_name(0, shape, 8, b, dtype, c16=mode == "c16").startswith("compress_strip<")
    _check_variant(shape, 8, b, mode)


# the block sizes of the sweep of Sec. 5 (12, 16, 18) on the small maps of a ResNet (28, 14 wide on ImageNet, 32, 16 on CIFAR):
# block rows of 12 or 18 rows are no DPP group, the strips' shares of a block meet in LDS
STRIP_SWEEP_CASES = [
    ((3, 171, 28, 28), 12, 2),          # 12 + 12 + 4 rows and columns, an odd number of planes
    ((2, 33, 28, 28), 18, 4),           # 18 + 10
    ((2, 33, 28, 28), 16, 8),           # 16 + 12: block rows of 16 lanes
    ((3, 67, 32, 32), 12, 2),           # 12 + 12 + 8, every lane slot in use
    ((3, 67, 32, 32), 18, 4),           # 18 + 14
    ((2, 33, 32, 32), 16, 2),
    ((5, 41, 16, 16), 12, 2),           # 12 + 4, two rows per lane, 205 planes in rounds of 8
    ((5, 41, 14, 14), 12, 8),           # 12 + 2
    ((3, 67, 20, 28), 12, 2),           # 12 + 8 rows
    ((3, 67, 13, 32), 12, 4),           # 12 + 1 rows
    ((3, 67, 30, 32), 18, 2),           # 18 + 12 rows
    ((3, 67, 19, 28), 18, 2),           # 18 + 1 rows
    ((3, 67, 6, 16), 12, 2),            # one block row of 6 rows
    ((3, 67, 14, 16), 12, 4),           # 12 + 2 rows, two per lane
    ((1, 1, 32, 32), 18, 2), ((1, 1, 16, 16), 12, 2),
    ((9, 600, 16, 16), 12, 2),          # 5400 planes: more than one run of the XCD-aware order and its plain tail
    # B = 4 and 8 on the CIFAR widths: block rows of 4 / 8 rows are DPP groups of 4, 2 (two rows per lane) or 8 lanes
    ((3, 67, 32, 32), 4, 2),            # 8 x 8 blocks: eight block columns per strip
    ((3, 67, 32, 32), 8, 4),
    ((5, 41, 16, 16), 4, 8),            # groups of two lanes
    ((5, 41, 16, 16), 8, 2),
    ((3, 67, 30, 32), 4, 2),            # ragged last block row (2 of 4 rows)
    ((3, 67, 27, 32), 8, 2),            # 3 of 8 rows
    ((3, 67, 10, 16), 4, 4),            # 2 of 4 rows, two rows per lane
    ((3, 67, 12, 16), 8, 2),
]


@pytest.mark.parametrize("shape,B,b", STRIP_SWEEP_CASES)
@pytest.mark.parametrize("mode", ["f32", "bf16", "c16"])
def test_strip_kernel_under_the_block_sizes_of_the_sweep(shape, B, b, mode):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    name = pkg.division_kernel_name(0, shape, B, b, dtype, c16=mode == "c16")
    assert name.startswith("compress_strip<") and name.endswith(", %d, %d>" % (shape[3], B)), name
    _check_variant(shape, B, b, mode)


# planes of an odd width (13, 15, 17, 27, 35, 55): a row per lane, rows that start in the middle of an element pair
ROWSTRIP_CASES = [
    ((3, 5, 13, 13), 8), ((7, 9, 13, 13), 4), ((5, 3, 15, 15), 8), ((5, 3, 15, 15), 4), ((3, 5, 17, 17), 8), ((2, 3, 27, 27), 8),
    ((3, 5, 9, 13), 8),                  # 8 + 1 rows
    ((3, 5, 16, 13), 4),                 # every lane slot in use
    ((3, 5, 2, 15), 8), ((3, 5, 3, 17), 8),
    ((3, 5, 32, 27), 8),                 # every lane slot in use, 32 rows
    ((3, 5, 31, 17), 8),
    ((1, 1, 13, 13), 8), ((1, 1, 27, 27), 8),
    ((1, 7, 27, 27), 8), ((3, 67, 13, 13), 8),     # rounds that end before their last plane slot
    ((2, 3, 35, 35), 8), ((2, 3, 55, 55), 8), ((2, 3, 55, 55), 4),       # a plane per wavefront
    ((3, 5, 17, 17), 4), ((2, 3, 27, 27), 4), ((2, 3, 35, 35), 4), ((2, 3, 30, 27), 4), ((1, 3, 63, 35), 4),
    ((1, 3, 64, 35), 8), ((1, 2, 40, 55), 4), ((1, 1, 55, 55), 8), ((1, 2, 5, 55), 8),
    ((9, 600, 15, 15), 8),               # 5400 planes: more than one run of the XCD-aware order and its plain tail
]


@pytest.mark.parametrize("shape,B", ROWSTRIP_CASES)
@pytest.mark.parametrize("b", [1, 2, 4, 8])
@pytest.mark.parametrize("mode", ["f32", "bf16", "c16"])
def test_row_per_lane_kernel_on_odd_widths(shape, B, b, mode):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    c16 = mode == "c16"
    name = pkg.division_kernel_name(0, shape, B, b, dtype, c16=c16)
    assert name.startswith("compress_rowstrip<") and name.endswith(", %d, %d, %d>" % (b, shape[3], B)), name
    _check_variant(shape, B, b, mode)
    # code words of a buffer that held something else before: every bit is written, pad bits are zero
    dt = oracle.F32_C16 if c16 else (oracle.BF16 if mode == "bf16" else oracle.F32)
    x = _relu_normal(shape, 11 + B + b, dtype)
    xh, _ = to_host_array(x)
    pk = torch.full((pkg.division_packed_bytes(*shape, B, b, dtype, c16),), 0xFF, dtype=torch.uint8, device="cuda:0")
    pkg.division_compress(x.to("cuda:0"), B, b, 4242, packed=pk, c16=c16)
    torch.cuda.synchronize()
    assert np.array_equal(pk.cpu().numpy(), oracle.compress(xh, B, b, 4242, dt, threads=16))


@pytest.mark.parametrize("shape,B,b", ROWS_CASES)
@pytest.mark.parametrize("mode", ["f32", "bf16", "c16"])
def test_general_block_size_kernel_matches_oracle(shape, B, b, mode):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    c16 = mode == "c16"
    name = pkg.division_kernel_name(0, shape, B, b, dtype, c16=c16)
    # block sizes 12 and 16 on planes of whole 4-element units take the register kernel's any-B instance
    # (1-D maps with power-of-two blocks the one-row kernel), other planes of 256 elements and more
    # the register kernel for any width
    units = shape[2] > 1 and shape[2] * shape[3] >= 256
    assert (name.startswith(("compress_rows<", "compress_line<", "compress_strip<")) or (name.startswith("compress_regs<") and ", 0, " in name)
            or (units and name.startswith("compress_units<")))
    _check_variant(shape, B, b, mode)


# image-sized planes (13 K - 53 K elements) in the registers of a 1024-thread workgroup
BIG_REGS_CASES = [
    ((2, 3, 224, 224), 8, 2),           # 12544 units: 13 per lane but the last round
    ((2, 2, 200, 200), 8, 4),           # 25 x 25 blocks
    ((1, 3, 160, 168), 4, 8),           # B = 4: 1680 blocks
    ((2, 2, 128, 128), 8, 2),           # 4096 units: four rounds
    ((1, 2, 228, 232), 8, 2),           # 13224 units: nearly full; ragged blocks both ways
]


@pytest.mark.parametrize("shape,B,b", BIG_REGS_CASES)
@pytest.mark.parametrize("mode", ["f32", "bf16", "c16"])
def test_register_kernel_with_1024_threads_matches_oracle(shape, B, b, mode):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    name = pkg.division_kernel_name(0, shape, B, b, dtype, c16=mode == "c16")
    assert name.startswith("compress_regs<") and name.endswith(", 16>")
    _check_variant(shape, B, b, mode)


# the register kernel's instance for any block size that is a multiple of 4 (up to 16)
REGS_ANY_CASES = [
    ((4, 6, 40, 52), 12, 2),            # 520 units, blocks of 12 and 4 both ways
    ((3, 4, 64, 64), 16, 4),            # 1024 units: four wavefronts, full blocks
    ((2, 5, 48, 44), 12, 8),            # 528 units: rounds of units past the plane are skipped
    ((5, 3, 48, 48), 12, 2),            # full blocks of 12
    ((9, 2, 56, 56), 16, 2),            # blocks 16, 16, 16, 8
    ((2, 2, 112, 112), 12, 4),          # 3136 units, 100 blocks
    ((3, 2, 24, 100), 16, 2),
    ((3, 5, 1, 3072), 64, 2),           # 1-D map, blocks of 64 elements (16 units)
    ((2, 4, 2, 2048), 64, 4),           # two rows: 32 units per block
    ((3, 3, 1, 2400), 32, 8),           # 75 blocks of 32
    ((2, 3, 1, 2100), 64, 2),           # ragged last block of 52
]


@pytest.mark.parametrize("shape,B,b", REGS_ANY_CASES)
@pytest.mark.parametrize("mode", ["f32", "bf16", "c16"])
def test_register_kernel_any_block_size_matches_oracle(shape, B, b, mode):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    name = pkg.division_kernel_name(0, shape, B, b, dtype, c16=mode == "c16")
    one_row_bf16 = shape[2] == 1 and mode == "bf16"            # 2-byte 1-D maps go to the one-row kernel first
    assert (name.startswith("compress_regs<") and ", 0, " in name) or (one_row_bf16 and name.startswith("compress_line<"))
    _check_variant(shape, B, b, mode)


# planes whose rows or blocks are not whole 16-byte vectors: the register kernel with a block per element
UNITS_CASES = [
    ((2, 3, 57, 57), 8, 2),             # 813 units (the last one holds one element), two wavefronts
    ((3, 2, 53, 53), 4, 4),             # 742 row segments of 4 (1 at the right edge)
    ((3, 5, 29, 29), 8, 2),             # 211 units: one wavefront, four rounds
    ((2, 3, 29, 29), 4, 8),
    ((2, 2, 147, 147), 8, 2),           # 5403 units: sixteen wavefronts
    ((1, 3, 149, 149), 4, 4),           # 5476 row segments
    ((2, 2, 73, 73), 8, 4),             # 1333 units: four wavefronts
    ((2, 3, 35, 35), 3, 2),             # B = 3: 432 row segments, blocks of 3 and 2
    ((2, 3, 56, 56), 18, 2),            # rows of whole vectors, blocks of 18, 18, 18, 2
    ((3, 2, 57, 57), 12, 8),
    ((2, 2, 30, 34), 18, 2),            # even width that is not a multiple of 4
    ((2, 2, 163, 163), 8, 2),           # 6643 units, 143 KB of LDS: about the largest plane the kernel takes
    ((2, 2, 33, 61), 5, 4),
    ((4, 3, 23, 23), 64, 2),            # one block per plane with an odd element count
    ((3, 3, 26, 45), 8, 2),             # odd width, even element count: 2-byte planes start on 4-byte boundaries
    ((2, 3, 38, 75), 4, 4),             # H*W % 4 == 2: the last unit holds two elements
    ((6, 5, 19, 19), 8, 2),             # planes below 512 elements: 16 lanes per plane, four planes per wavefront;
    ((5, 7, 19, 19), 4, 4),             # 30 planes: the last round has two
    ((3, 3, 21, 21), 2, 8),             # 242 row segments: 32 lanes per plane
    ((4, 6, 17, 17), 18, 2),            # one block per plane
    ((7, 3, 17, 23), 6, 2),
    ((1, 1, 57, 57), 8, 2),             # a single plane
    ((2, 2, 2, 1001), 8, 4),            # two long rows: 126 blocks in one block row
    ((1, 3, 127, 129), 8, 2),           # 16383 elements: eight wavefronts
    ((3, 1, 3, 4099), 8, 2),            # 513 blocks of 3 rows: 4104 row segments
    ((2, 2, 3000, 3), 8, 2),            # rows shorter than a unit: a unit spans two rows
    ((1, 2, 1000, 5), 4, 4),
]


@pytest.mark.parametrize("shape,B,b", UNITS_CASES)
@pytest.mark.parametrize("mode", ["f32", "bf16", "c16"])
def test_register_kernel_any_width_matches_oracle(shape, B, b, mode):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    assert pkg.division_kernel_name(0, shape, B, b, dtype, c16=mode == "c16").startswith("compress_units<")
    if shape[3] % 2 == 1 and shape[2] * shape[3] >= 512:      # (smaller planes are rebuilt chunk-wise in LDS)
        # (4-byte elements: the wavefront-per-chunk kernel for any width where a plane has several blocks of 4 and more)
        assert pkg.division_kernel_name(1, shape, B, b, dtype, c16=mode == "c16").startswith(("decompress_units<", "decompress_stream_any<", "decompress_stream_one<"))
    _check_variant(shape, B, b, mode)


# more planes than workgroups: a workgroup takes every grid-th plane, the next one's loads in flight
@pytest.mark.parametrize("shape,B,b", [((21, 100, 57, 57), 8, 2), ((3, 100, 147, 147), 8, 2), ((42, 100, 29, 29), 4, 4),
                                        ((3, 1001, 37, 37), 8, 2), ((5, 4001, 19, 19), 8, 2)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_register_kernel_any_width_many_planes(shape, B, b, dtype):
    assert pkg.division_kernel_name(0, shape, B, b, dtype).startswith("compress_units<")
    x = _relu_normal(shape, 4242 + shape[1], dtype)
    xh, _ = to_host_array(x)
    dt = oracle.BF16 if dtype == torch.bfloat16 else oracle.F32
    ref = oracle.compress(xh, B, b, 99, dt, threads=16)
    pk = pkg.division_compress(x.to("cuda:0"), B, b, 99)
    y = pkg.division_decompress(pk, shape, B, b, dtype)
    torch.cuda.synchronize()
    assert np.array_equal(pk.cpu().numpy(), ref)
    yh, _ = to_host_array(y.cpu())
    assert np.array_equal(yh, oracle.decompress(ref, shape, B, b, dt))


def _check_variant(shape, B, b, mode):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    c16 = mode == "c16"
    g = torch.Generator().manual_seed(7000 + sum(shape) + 13 * B + b)
    x = (torch.randn(shape, generator=g) * 2.0 + 0.25).to(dtype)       # signed values
    x[0, 0] = 1.5                                                     # one constant plane (degenerate scale)
    dt = oracle.F32_C16 if c16 else (oracle.BF16 if mode == "bf16" else oracle.F32)
    xh, _ = to_host_array(x)
    seed = 0x0B10C5 + B
    ref = oracle.compress(xh, B, b, seed, dt, threads=16)
    xd = x.to("cuda:0")
    pk = pkg.division_compress(xd, B, b, seed, c16=c16)
    y = pkg.division_decompress(pk, shape, B, b, dtype, c16=c16)
    pb = pkg.division_compress_batch([xd, xd, xd], B, b, [seed + 1, seed, seed + 2], c16=c16)
    torch.cuda.synchronize()
    assert np.array_equal(pk.cpu().numpy(), ref)
    assert torch.equal(pb[1], pk)
    assert np.array_equal(pb[2].cpu().numpy(), oracle.compress(xh, B, b, seed + 2, dt, threads=16))
    yh, _ = to_host_array(y.cpu())
    assert np.array_equal(yh, oracle.decompress(ref, shape, B, b, dt))


# ---------------------------------------------------------------- the paper's cached format (bfloat16 H^L, delta, Delta)

C16_CASES = [
    ((3, 5, 56, 56), 8, 2), ((2, 2, 96, 96), 8, 4), ((4, 7, 28, 28), 8, 2), ((5, 9, 14, 14), 8, 2), ((37, 9, 7, 7), 8, 2),
    ((2, 3, 72, 72), 8, 2), ((2, 3, 55, 55), 4, 4), ((2, 3, 36, 36), 12, 2), ((3, 4, 32, 32), 4, 8), ((2, 2, 9, 6), 4, 2),
    ((1, 2, 300, 300), 8, 2), ((2, 3, 50, 44), 8, 4), ((40, 13, 4, 4), 4, 2), ((3, 5, 1, 197), 8, 2), ((300, 7, 7, 7), 8, 4),
    ((2, 3, 64, 64), 8, 2), ((5, 4, 1, 50), 64, 2), ((1, 1, 1, 1), 4, 2),
]


@pytest.mark.parametrize("shape,B,b", C16_CASES)
@pytest.mark.parametrize("kind", ["relu", "signed_large"])
def test_bfloat16_cached_mode_matches_oracle(shape, B, b, kind):
    x = _relu_normal(shape, 5000 + sum(shape) + B + b)
    if kind == "signed_large":
        g = torch.Generator().manual_seed(sum(shape))
        x = torch.randn(shape, generator=g) * 300.0 - 1000.0        # negative minima, large bfloat16 steps
    seed = 0x5EED0000 + B
    ref = oracle.compress(x.numpy(), B, b, seed, oracle.F32_C16)
    xd = x.to("cuda:0")
    need = pkg.division_packed_bytes(*shape, B, b, c16=True)
    assert need == ref.size
    pk = torch.full((need,), 0x5A, dtype=torch.uint8, device="cuda:0")
    pkg.division_compress(xd, B, b, seed, packed=pk, c16=True)
    y = pkg.division_decompress(pk, shape, B, b, c16=True)
    pb = pkg.division_compress_batch([xd, xd], B, b, [seed, seed + 7], c16=True)
    yb = pkg.division_decompress_batch(pb, shape, B, b, c16=True)
    torch.cuda.synchronize()
    assert np.array_equal(pk.cpu().numpy(), ref)
    assert np.array_equal(y.cpu().numpy(), oracle.decompress(ref, shape, B, b, oracle.F32_C16))
    assert torch.equal(pb[0], pk) and torch.equal(yb[0], y)
    assert np.array_equal(pb[1].cpu().numpy(), oracle.compress(x.numpy(), B, b, seed + 7, oracle.F32_C16))


def test_bfloat16_cached_mode_full_size_resnet50_set():
    total_in = total_pk = 0
    for k, spec, x in draw_config(2):
        seed = codec_seed(2, k)
        ref = oracle.compress(x.numpy(), spec.B, spec.b, seed, oracle.F32_C16, threads=16)
        pk = pkg.division_compress(x.to("cuda:0"), spec.B, spec.b, seed, c16=True)
        y = pkg.division_decompress(pk, tuple(x.shape), spec.B, spec.b, c16=True)
        torch.cuda.synchronize()
        assert np.array_equal(pk.cpu().numpy(), ref), spec.name
        assert np.array_equal(y.cpu().numpy(), oracle.decompress(ref, tuple(x.shape), spec.B, spec.b, oracle.F32_C16, threads=16))
        total_in += x.numel() * 4
        total_pk += pk.numel()
        del pk, y
    assert total_in / total_pk > 12.0          # 12.2x against 11.5x with fp32 H^L and (delta, Delta)


# ---------------------------------------------------------------- byte offsets beyond 4 GiB

@pytest.mark.parametrize("shape,B,b", [((1400, 256, 56, 56), 8, 2), ((1100, 1024, 32, 32), 4, 4), ((3700, 96, 55, 55), 4, 2)])
def test_full_size_maps_larger_than_4GiB(shape, B, b):
    """1.1 G elements (4.5 GB of fp32): plane offsets in bytes and in elements pass 2^32 resp. 2^30;
    the last planes are the ones a 32-bit index would send elsewhere."""
    g = torch.Generator(device="cuda:0").manual_seed(77)
    xd = torch.relu(torch.randn(shape, generator=g, device="cuda:0"))
    x = xd.cpu().numpy()
    seed = 0xB16B00B5
    pk = pkg.division_compress(xd, B, b, seed)
    torch.cuda.synchronize()
    ref = oracle.compress(x, B, b, seed, threads=16)
    assert np.array_equal(pk.cpu().numpy(), ref)
    del ref
    y = pkg.division_decompress(pk, shape, B, b)
    torch.cuda.synchronize()
    yr = oracle.decompress(pk.cpu().numpy(), shape, B, b, threads=16)
    assert np.array_equal(y.cpu().numpy(), yr)


# ---------------------------------------------------------------- values at the edges of binary32, under every kernel family

SPECIAL_VALUE_SHAPES = [
    ((3, 4, 56, 56), 8), ((3, 4, 28, 28), 8), ((3, 4, 14, 14), 8), ((6, 2, 7, 7), 8), ((3, 4, 4, 4), 4),
    ((3, 4, 55, 55), 8), ((2, 6, 17, 17), 4), ((3, 4, 28, 28), 12), ((3, 4, 54, 57), 64), ((3, 4, 56, 56), 64),
    ((3, 4, 1, 196), 16), ((2, 6, 96, 96), 8), ((3, 4, 150, 150), 18), ((3, 4, 27, 35), 5), ((4, 3, 32, 32), 4),
    ((3, 4, 13, 13), 8), ((3, 4, 30, 30), 4), ((1, 12, 300, 300), 18), ((3, 4, 56, 56), 12), ((3, 4, 170, 170), 8),
    ((3, 4, 250, 250), 8), ((3, 4, 60, 60), 8), ((3, 4, 224, 224), 8), ((2, 6, 9, 6), 4), ((3, 4, 1, 3072), 4096),
    ((3, 4, 27, 27), 8), ((3, 4, 17, 17), 8), ((3, 4, 15, 15), 4),
]


def _special_planes(shape, seed):
    """Thirteen planes (repeated over the tensor) that sit at the edges of the arithmetic: zero and constant planes,
    an outlier, subnormal values, residual ranges below and just above the degenerate threshold, a residual range
    that overflows binary32 although every residual is finite, negative zeros, a large offset with small variation."""
    N, C, H, W = shape
    g = torch.Generator().manual_seed(seed)
    r = lambda: torch.randn((H, W), generator=g)
    half = torch.arange(H * W).view(H, W) * 2 < H * W
    sign = torch.where(torch.rand((H, W), generator=g) < torch.where(half, 0.25, 0.75), 1.0, -1.0)
    planes = [
        torch.zeros(H, W),
        torch.full((H, W), 3.25),
        torch.where(torch.arange(H * W).view(H, W) == (H * W) // 3, 1e30, 1.0) * r(),
        r() * 1e-41,                                   # subnormal values: sums and means stay subnormal
        r() * 1e-30,                                   # residual range below 2^-90
        r() * 1e-26,                                   # just above it: scale factors near 2^86
        sign * 1.6e38,                                 # |residual| <= 3.2e38, range beyond the largest binary32
        -torch.zeros(H, W),
        torch.where(r() > 1.0, 1e-45, 1.0) * r(),      # subnormal and ordinary values in one plane
        1e3 + r() * 1e-2,
        torch.where(r() > 0, 2.5, -7.0),               # two values only
        r().clamp_min(0),
        # +-a on a checkerboard, a = 1.99609375 * 2^126: block means 0 (even blocks), the residual range is finite but
        # beyond the largest bfloat16, which a 1-bit step in the bfloat16-cached format would have to hold
        torch.where((torch.arange(H).view(H, 1) + torch.arange(W).view(1, W)) % 2 == 0, 1.0, -1.0) * (1.99609375 * 2.0 ** 126),
    ]
    x = torch.stack([planes[i % len(planes)] for i in range(N * C)]).view(shape)
    return x.contiguous()


@pytest.mark.parametrize("shape,B", SPECIAL_VALUE_SHAPES)
@pytest.mark.parametrize("mode,b", [("f32", 2), ("f32", 8), ("bf16", 4), ("c16", 2), ("f32", 1), ("bf16", 1), ("c16", 1)])
def test_values_at_the_edges_of_binary32(shape, B, mode, b):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    c16 = mode == "c16"
    dt = oracle.F32_C16 if c16 else (oracle.BF16 if mode == "bf16" else oracle.F32)
    x = _special_planes(shape, 31 + B).to(dtype)
    xh, _ = to_host_array(x)
    ref = oracle.compress(xh, B, b, 2024, dt, threads=16)
    pk = pkg.division_compress(x.to("cuda:0"), B, b, 2024, c16=c16)
    y = pkg.division_decompress(pk, shape, B, b, dtype, c16=c16)
    torch.cuda.synchronize()
    got = pk.cpu().numpy()
    if not np.array_equal(got, ref):
        s, t = oracle.split_packed(got, shape, B, b, dt), oracle.split_packed(ref, shape, B, b, dt)
        where = {k: sorted({int(i) % 13 for i in np.nonzero(s[k].reshape(s[k].shape[0], -1).view(np.uint8)
                                                           != t[k].reshape(t[k].shape[0], -1).view(np.uint8))[0]})
                 for k in ("lfc", "meta", "codes")}
        raise AssertionError(f"{pkg.division_kernel_name(0, shape, B, b, dtype, c16=c16)}: kinds of plane that differ {where}")
    yh, _ = to_host_array(y.cpu())
    assert np.array_equal(yh, oracle.decompress(ref, shape, B, b, dt), equal_nan=mode != "bf16")


@pytest.mark.parametrize("shape,B", SPECIAL_VALUE_SHAPES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_a_plane_of_nan_and_infinity_leaves_the_other_planes_alone(shape, B, dtype):
    # what such a plane is compressed to is unspecified; its neighbours (same wavefront, same workgroup) must not see it
    N, C, H, W = shape
    x = _relu_normal(shape, 77 + B, dtype)
    xp = x.view(N * C, -1)
    bad = [1, N * C // 2, N * C - 1]
    g = torch.Generator().manual_seed(B)
    for i, p in enumerate(bad):
        r = torch.randn(H * W, generator=g)
        xp[p] = [torch.full_like(r, float("nan")), torch.where(r > 0, float("inf"), -float("inf")),
                 torch.where(r > 1, float("nan"), r)][i].to(dtype)
    xh, dt = to_host_array(x)
    ref = oracle.split_packed(oracle.compress(xh, B, 4, 6, dt, threads=16), shape, B, 4, dt)
    pk = pkg.division_compress(x.to("cuda:0"), B, 4, 6)
    y = pkg.division_decompress(pk, shape, B, 4, dtype)
    torch.cuda.synchronize()
    got = oracle.split_packed(pk.cpu().numpy(), shape, B, 4, dt)
    good = np.setdiff1d(np.arange(N * C), bad)
    for k in ("codes", "meta", "lfc"):
        a, r_ = got[k].reshape(N * C, -1), ref[k].reshape(N * C, -1)
        assert np.array_equal(a[good].view(np.uint8), r_[good].view(np.uint8)), k
    yh, _ = to_host_array(y.cpu())
    want = oracle.decompress(pk.cpu().numpy(), shape, B, 4, dt).reshape(N * C, -1)
    assert np.array_equal(yh.reshape(N * C, -1)[good], want[good])


# planes of 10^5 .. 2 x 10^6 elements and block sizes from 3 to far beyond the map: the general kernels' index arithmetic
@pytest.mark.parametrize("shape,B", [((2, 3, 1, 100003), 8), ((2, 3, 1, 100003), 1000), ((2, 3, 1, 100003), 1 << 20),
                                      ((2, 3, 1, 1 << 20), 4096), ((2, 3, 1, 1 << 20), 65536), ((1, 2, 1, 65537 * 4), 100003),
                                      ((1, 2, 1031, 1033), 8), ((1, 2, 1031, 1033), 2000), ((1, 2, 1024, 1024), 128),
                                      ((1, 1, 4099, 257), 4099), ((1, 2, 257, 4100), 3), ((1, 1, 2, 500001), 1024),
                                      ((1, 1, 500001, 2), 8), ((1, 1, 70001, 1), 70000), ((1, 2, 3, 3, 40000), 128),
                                      ((1, 2, 40000, 3, 3), 2000), ((1, 1, 130, 130, 130), 8), ((1, 1, 130, 130, 130), 4099)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_long_maps_and_blocks_far_larger_than_the_map(shape, B, dtype):
    three = len(shape) == 5
    b = 2 if B % 2 == 0 else 4
    x = _relu_normal(shape, B + sum(shape), dtype)
    xh, dt = to_host_array(x)
    ref = oracle.compress(xh, B, b, 9, dt, threads=16)
    pk = (pkg.division_compress_3d if three else pkg.division_compress)(x.to("cuda:0"), B, b, 9)
    y = (pkg.division_decompress_3d if three else pkg.division_decompress)(pk, shape, B, b, dtype)
    torch.cuda.synchronize()
    assert np.array_equal(pk.cpu().numpy(), ref)
    yh, _ = to_host_array(y.cpu())
    assert np.array_equal(yh, oracle.decompress(ref, shape, B, b, dt, threads=16))


# maps and outputs that start 1, 2, 3 or 5 elements past a 16-byte boundary, with guard elements on both sides of the output
# and guard bytes behind the packed buffer
@pytest.mark.parametrize("shape,B", SPECIAL_VALUE_SHAPES + [((2, 6, 5, 9, 13), 4), ((1, 12, 4, 28, 28), 8), ((2, 6, 8, 27, 27), 8),
                                                             ((1, 12, 16, 16, 16), 8)])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_unaligned_maps_and_outputs_under_every_kernel_family(shape, B, dtype):
    three = len(shape) == 5
    numel, pad, guard = int(np.prod(shape)), 64, 7.0
    compress = pkg.division_compress_3d if three else pkg.division_compress
    decompress = pkg.division_decompress_3d if three else pkg.division_decompress
    for off in (1, 2, 3, 5):
        x = _relu_normal(shape, B + sum(shape) + off, dtype)
        xh, dt = to_host_array(x)
        ref = oracle.compress(xh, B, 2, 9, dt, threads=16)
        base = torch.zeros(numel + 2 * pad, dtype=dtype, device="cuda:0")
        base[pad + off: pad + off + numel] = x.flatten().to("cuda:0")
        big = torch.full((ref.size + 256,), 0x5A, dtype=torch.uint8, device="cuda:0")      # guard bytes behind the packed buffer
        compress(base[pad + off: pad + off + numel].view(shape), B, 2, 9, packed=big)
        pk = big[:ref.size]
        ob = torch.full((numel + 2 * pad,), guard, dtype=dtype, device="cuda:0")
        decompress(pk, shape, B, 2, dtype, out=ob[pad + off: pad + off + numel].view(shape))
        torch.cuda.synchronize()
        assert np.array_equal(pk.cpu().numpy(), ref) and bool((big[ref.size:] == 0x5A).all()), off
        obh = ob.cpu()
        yh, _ = to_host_array(obh[pad + off: pad + off + numel].contiguous())
        assert np.array_equal(yh.reshape(shape), oracle.decompress(ref, shape, B, 2, dt, threads=16)), off
        assert bool((obh[:pad + off] == guard).all()) and bool((obh[pad + off + numel:] == guard).all()), off


# fp32 maps whose rows and planes are not whole 16-byte vectors, rebuilt by the wavefront-per-chunk kernel: the element
# count of the map leaves 1, 2 or 3 elements in its last vector, planes end inside vectors, chunks end inside planes
STREAM_ANY_CASES = [
    ((1, 1, 13, 13), 8, 2), ((1, 2, 13, 13), 8, 4), ((1, 3, 13, 13), 4, 8), ((3, 5, 17, 17), 8, 2), ((2, 3, 55, 55), 8, 2),
    ((7, 11, 27, 27), 8, 1), ((2, 3, 147, 147), 8, 2), ((5, 7, 3, 5), 4, 2), ((9, 9, 1, 9), 4, 4), ((3, 7, 2, 5), 4, 2),
    ((2, 3, 30, 35), 5, 2), ((3, 5, 1, 197), 8, 2), ((2, 2, 1, 4099), 64, 2), ((40, 25, 5, 7), 4, 2), ((2, 3, 57, 57), 7, 2),
    ((2, 2, 3, 9, 11), 4, 2), ((2, 2, 3, 35, 35), 4, 4), ((5, 3, 4, 9, 9), 8, 2), ((3, 2, 5, 7, 7), 4, 1), ((2, 3, 7, 5, 30), 5, 2),
]


# the same for planes that are one block: H^L is the plane's
STREAM_ONE_CASES = [
    ((5, 7, 9, 9), 16, 2), ((3, 67, 7, 10), 16, 4), ((37, 9, 11, 11), 64, 1), ((2, 3, 14, 14), 64, 2), ((3, 5, 16, 16), 18, 8),
    ((4, 3, 23, 23), 64, 2), ((2, 3, 2, 2), 8, 2), ((9, 5, 1, 50), 64, 4), ((1, 1, 1, 6), 8, 2), ((1, 3, 1, 70), 128, 2),
    ((7, 9, 5, 6), 8, 2), ((4, 9, 3, 3, 6), 8, 2), ((3, 4, 2, 4, 6), 8, 4),
]


@pytest.mark.parametrize("shape,B,b", STREAM_ANY_CASES + STREAM_ONE_CASES)
@pytest.mark.parametrize("mode", ["f32", "c16"])
def test_wavefront_per_chunk_decompress_of_any_width(shape, B, b, mode):
    three = len(shape) == 5
    c16 = mode == "c16"
    dt = oracle.F32_C16 if c16 else oracle.F32
    name = (pkg.division_kernel_name_3d if three else pkg.division_kernel_name)(1, shape, B, b, torch.float32, c16=c16)
    assert name.startswith("decompress_stream_one" if (shape, B, b) in STREAM_ONE_CASES else "decompress_stream_any"), name
    numel, guard = int(np.prod(shape)), -777.0
    g = torch.Generator().manual_seed(sum(shape) + B + b)
    x = (torch.randn(shape, generator=g) * 1.5 + 0.2)
    ref = oracle.compress(x.numpy(), B, b, 31337, dt, threads=16)
    ob = torch.full((numel + 64,), guard, dtype=torch.float32, device="cuda:0")           # guard elements behind the map
    out = ob[:numel].view(shape)
    (pkg.division_decompress_3d if three else pkg.division_decompress)(torch.from_numpy(ref).to("cuda:0"), shape, B, b, torch.float32, out=out, c16=c16)
    torch.cuda.synchronize()
    obh = ob.cpu().numpy()
    assert np.array_equal(obh[:numel].reshape(shape), oracle.decompress(ref, shape, B, b, dt, threads=16))
    assert (obh[numel:] == guard).all()


@pytest.mark.parametrize("seed", [0, 1, 2 ** 32, 2 ** 32 - 1, 2 ** 63 + 5, 2 ** 64 - 1])
def test_seeds_over_the_whole_64_bit_range(seed):
    # both halves of the seed reach the stream (Eq. quantization's rounding draws), in single and in batch calls
    shapes = [((3, 4, 28, 28), 8), ((2, 3, 55, 55), 4), ((5, 2, 7, 7), 8)]
    for shape, B in shapes:
        x = _relu_normal(shape, 5 + B)
        ref = oracle.compress(x.numpy(), B, 4, seed)
        xd = x.to("cuda:0")
        pk = pkg.division_compress(xd, B, 4, seed)
        pb = pkg.division_compress_batch([xd, xd], B, 4, [seed ^ 1, seed])
        torch.cuda.synchronize()
        assert np.array_equal(pk.cpu().numpy(), ref)
        assert torch.equal(pb[1], pk) and not torch.equal(pb[0], pk)
