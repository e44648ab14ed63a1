"""GPU parity of the 1-bit mask operators (Relu / Dropout) against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2208_04187_amd as pkg

pytestmark = pytest.mark.gpu

SIZES = [1, 3, 31, 32, 33, 255, 256, 1000, 4096, 4097, 65536 + 7, (1 << 20) + 5, 3 * 64 * 56 * 56]


def _values(n, seed, dtype):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(n, generator=g)
    x[::7] = 0.0
    x[3::11] = -0.0
    if n > 40:
        x[5] = float("nan"); x[6] = float("inf"); x[8] = -float("inf"); x[9] = 1e-45
    return x.to(dtype)


def _host(t: torch.Tensor):
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).numpy().view(np.uint16), oracle.BF16
    return t.contiguous().numpy(), oracle.F32


def _same_bits(a: torch.Tensor, ref: np.ndarray):
    h, _ = _host(a.cpu())
    return np.array_equal(h.view(np.uint16 if h.dtype == np.uint16 else np.uint32), ref.view(np.uint16 if ref.dtype == np.uint16 else np.uint32))


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_relu_forward_and_backward_match_oracle(n, dtype):
    x = _values(n, 100 + n % 97, dtype)
    g = _values(n, 200 + n % 89, dtype)
    xh, dt = _host(x)
    gh, _ = _host(g)
    y_ref, m_ref = oracle.relu_forward(xh, dt)
    y, m = pkg.division_relu_forward(x.to("cuda:0"))
    torch.cuda.synchronize()
    assert np.array_equal(m.cpu().numpy().view(np.uint32), m_ref)
    assert _same_bits(y, y_ref)
    gin = pkg.division_mask_backward(m, g.to("cuda:0"))
    torch.cuda.synchronize()
    assert _same_bits(gin, oracle.mask_backward(m_ref, gh, dt))


# the last two: p * 65536 + 1/2 is 2^-25 below 1 (T = 0: nothing dropped, also where r == 0) and exactly 1 (T = 1)
@pytest.mark.parametrize("p", [0.0, 0.1, 0.5, 0.9, 1.0, (0.5 - 2.0 ** -25) / 65536, 0.5 / 65536])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_dropout_forward_matches_oracle(p, dtype):
    for n, seed in ((1, 1), (77, 2), (4097, 0xFEDCBA9876543210), ((1 << 19) + 3, 4)):
        x = _values(n, 300 + n % 83, dtype)
        xh, dt = _host(x)
        y_ref, m_ref = oracle.dropout_forward(xh, p, seed, dt)
        y, m = pkg.division_dropout_forward(x.to("cuda:0"), p, seed)
        torch.cuda.synchronize()
        assert np.array_equal(m.cpu().numpy().view(np.uint32), m_ref)
        assert _same_bits(y, y_ref)


def test_unaligned_buffers_and_in_place():
    n = 5003
    base = torch.zeros(n + 3, device="cuda:0")
    x = _values(n, 9, torch.float32)
    base[3:].copy_(x)
    xd = base[3:]
    assert xd.data_ptr() % 16 != 0
    y_ref, m_ref = oracle.relu_forward(x.numpy())
    y, m = pkg.division_relu_forward(xd)
    torch.cuda.synchronize()
    assert np.array_equal(m.cpu().numpy().view(np.uint32), m_ref) and _same_bits(y, y_ref)
    # in place: y is x itself
    xa = x.to("cuda:0")
    y2, m2 = pkg.division_relu_forward(xa, out=xa)
    torch.cuda.synchronize()
    assert y2.data_ptr() == xa.data_ptr()
    assert np.array_equal(m2.cpu().numpy().view(np.uint32), m_ref) and _same_bits(xa, y_ref)
    g = _values(n, 10, torch.float32).to("cuda:0")
    ref = oracle.mask_backward(m_ref, g.cpu().numpy())
    pkg.division_mask_backward(m2, g, out=g)
    torch.cuda.synchronize()
    assert _same_bits(g, ref)


def test_mask_errors_and_empty_input():
    x = torch.zeros(100, device="cuda:0")
    small = torch.empty(3, dtype=torch.int32, device="cuda:0")
    with pytest.raises(pkg.DivisionError) as e:
        pkg.division_relu_forward(x, mask=small)
    assert e.value.code == 2
    y, m = pkg.division_relu_forward(torch.empty(0, device="cuda:0"))
    assert y.numel() == 0 and m.numel() == 0


# ---------------------------------------------------------------- Max-Pooling layer

MP_CASES = [((2, 3, 8, 8), 2), ((1, 2, 9, 7), 2), ((2, 2, 12, 9), 3), ((1, 1, 5, 5), 1), ((3, 1, 4, 6), 4),
            ((2, 5, 112, 112), 2), ((2, 1, 7, 7), 7), ((1, 1, 10, 13), 5), ((70, 33, 14, 14), 2),
            ((1, 1, 3, 3), 4), ((1, 2, 600, 300), 2), ((2, 3, 56, 56), 3),
            # k = 2 on rows of whole 8-element pieces: four windows per thread, mask bytes with one owner
            ((5, 7, 56, 56), 2), ((3, 2, 11, 32), 2),      # the second: an odd last row, written (as zeros) by the last band
            ((4, 3, 4, 8), 2), ((2, 2, 64, 40), 2), ((1, 2, 600, 304), 2), ((300, 9, 8, 16), 2),
            ((2, 3, 30, 24), 2), ((3, 2, 9, 16), 2)]        # H * W no multiple of 32: the general forward kernel, the fast backward one


@pytest.mark.parametrize("shape,k", MP_CASES)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_maxpool_matches_oracle(shape, k, dtype):
    g = torch.Generator().manual_seed(sum(shape) + k)
    x = torch.randn(shape, generator=g)
    x[..., ::3] = x[..., ::3].round()                 # plenty of ties, also across windows
    x = x.to(dtype)
    N, C, H, W = shape
    go = torch.randn((N, C, H // k, W // k), generator=g).to(dtype)
    xh, dt = _host(x)
    gh, _ = _host(go)
    y_ref, m_ref = oracle.maxpool_forward(xh, k, dt)
    y, m = pkg.division_maxpool_forward(x.to("cuda:0"), k)
    torch.cuda.synchronize()
    assert np.array_equal(m.cpu().numpy().view(np.uint32), m_ref)
    if y_ref.size:
        assert _same_bits(y, y_ref)
    gin = pkg.division_maxpool_backward(m, go.to("cuda:0"), shape, k)
    torch.cuda.synchronize()
    assert _same_bits(gin, oracle.maxpool_backward(m_ref, gh, shape, k, dt))


# ---------------------------------------------------------------- Relu fused with the compression of its output

@pytest.mark.parametrize("shape,B,b,fused", [
    ((3, 5, 56, 56), 8, 2, True),        # one wavefront per plane
    ((2, 3, 112, 112), 8, 4, True),      # four wavefronts per plane
    ((2, 4, 48, 48), 4, 8, True),        # B = 4, 2304 elements
    ((3, 4, 64, 32), 8, 2, True),        # 2048 elements
    ((2, 3, 50, 44), 8, 2, False),       # 2200 elements: not whole mask words per plane -> two kernels
    ((2, 3, 56, 56), 12, 2, False),      # block size outside the fused instances
    ((5, 9, 7, 7), 8, 4, False),         # lane-per-plane kernel -> two kernels
    ((2, 3, 30, 30), 4, 2, False),       # more than 64 pooling items per plane -> two kernels
    ((4, 7, 28, 28), 8, 2, True),        # strip kernel: two planes (1568 mask bits) per round
    ((3, 7, 28, 28), 8, 8, True),        # 21 planes: the last round holds one, its mask ends in half a word
    ((5, 9, 14, 14), 8, 2, True),        # eight planes per round, 45 planes: the last round holds five
    ((130, 3, 14, 14), 8, 4, True),      # 49 rounds
    ((3, 5, 12, 28), 8, 4, True),        # 28-wide, 12 rows: 672 bits per round
    ((3, 5, 30, 28), 8, 2, True),        # 28-wide, 30 rows: rounds are not whole mask words -> the items kernel
    ((7, 3, 6, 14), 8, 2, True),         # 14-wide, 6 rows, 21 planes
    ((3, 5, 32, 32), 8, 2, True),        # the CIFAR widths in the strip kernel: B = 8 and B = 4
    ((5, 3, 16, 16), 8, 4, True),
    ((3, 5, 20, 32), 4, 2, True),        # ragged: 20 rows
    ((3, 5, 10, 16), 4, 8, True),
    ((6, 5, 32, 32), 4, 2, True),        # CIFAR shapes: whole mask words per plane
    ((3, 7, 16, 16), 4, 8, True),
    ((5, 3, 8, 8), 4, 2, True),
    ((4, 5, 4, 4), 4, 2, True),          # one block per plane, 16 bits each
    ((7, 3, 10, 30), 8, 2, True),        # 300 bits per plane: four rounds of two planes per workgroup
    ((3, 3, 6, 10), 4, 2, True),         # 60 bits per plane
    ((2, 3, 30, 30), 8, 2, True),        # ragged blocks both ways
])
@pytest.mark.parametrize("mode", ["f32", "bf16", "c16"])
def test_relu_fused_with_compression_matches_relu_then_compress(shape, B, b, fused, mode):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    c16 = mode == "c16"
    dt = oracle.F32_C16 if c16 else (oracle.BF16 if mode == "bf16" else oracle.F32)
    rdt = oracle.BF16 if mode == "bf16" else oracle.F32
    assert pkg.division_relu_compress_fused(shape, B, b, dtype, c16) == fused
    g = torch.Generator().manual_seed(sum(shape) + B)
    x = (torch.randn(shape, generator=g) * 1.5).to(dtype)
    x[0, 0, 0, :4] = torch.tensor([0.0, -0.0, float("nan"), -1e-30]).to(dtype)
    xh = x.view(torch.int16).numpy().view(np.uint16) if mode == "bf16" else x.numpy()
    y_ref, m_ref = oracle.relu_forward(xh, rdt)
    seed = 0xFE11 + B
    p_ref = oracle.compress(y_ref.reshape(shape), B, b, seed, dt)
    xd = x.to("cuda:0")
    y, m, pk = pkg.division_relu_compress(xd, B, b, seed, c16=c16)
    torch.cuda.synchronize()
    yh = y.cpu().view(torch.int16).numpy().view(np.uint16) if mode == "bf16" else y.cpu().numpy()
    assert np.array_equal(yh.view(np.uint16 if mode == "bf16" else np.uint32), y_ref.reshape(shape).view(np.uint16 if mode == "bf16" else np.uint32))
    assert np.array_equal(m.cpu().numpy().view(np.uint32), m_ref)
    assert np.array_equal(pk.cpu().numpy(), p_ref)
    # in place, and the same bytes as the two separate calls
    x2 = xd.clone()
    y2, m2, pk2 = pkg.division_relu_compress(x2, B, b, seed, out=x2, c16=c16)
    y3, m3 = pkg.division_relu_forward(xd)
    pk3 = pkg.division_compress(y3, B, b, seed, c16=c16)
    torch.cuda.synchronize()
    assert torch.equal(pk2, pk) and torch.equal(m2, m) and torch.equal(pk3, pk) and torch.equal(m3, m)
    assert torch.equal(x2.view(torch.int16 if mode == "bf16" else torch.int32), y.view(torch.int16 if mode == "bf16" else torch.int32))


@pytest.mark.parametrize("shape,B", [((3, 4, 56, 56), 8), ((2, 6, 112, 112), 8), ((3, 4, 28, 28), 8), ((3, 4, 14, 14), 8),
                                      ((3, 4, 32, 32), 4), ((3, 4, 4, 4), 4), ((3, 4, 55, 55), 8), ((3, 4, 56, 56), 12)])
@pytest.mark.parametrize("mode,b", [("f32", 2), ("bf16", 4), ("c16", 8)])
def test_relu_fused_with_compression_on_values_at_the_edges_of_binary32(shape, B, mode, b):
    # zero, signed-zero, subnormal, near-degenerate and huge planes (and their negatives) through Relu and the codec
    from tests.test_gpu_parity import _special_planes
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    c16 = mode == "c16"
    dt = oracle.F32_C16 if c16 else (oracle.BF16 if mode == "bf16" else oracle.F32)
    rdt = oracle.BF16 if mode == "bf16" else oracle.F32
    x = _special_planes(shape, 91 + B)
    x[shape[0] // 2:] = -x[shape[0] // 2:]
    x = x.to(dtype)
    xh = x.view(torch.int16).numpy().view(np.uint16) if mode == "bf16" else x.numpy()
    y_ref, m_ref = oracle.relu_forward(xh, rdt)
    p_ref = oracle.compress(y_ref.reshape(shape), B, b, 515, dt)
    y, m, pk = pkg.division_relu_compress(x.to("cuda:0"), B, b, 515, c16=c16)
    torch.cuda.synchronize()
    bits = (torch.int16, np.uint16) if mode == "bf16" else (torch.int32, np.uint32)
    assert np.array_equal(y.cpu().view(bits[0]).numpy().view(bits[1]), y_ref.reshape(shape).view(bits[1]))
    assert np.array_equal(m.cpu().numpy().view(np.uint32), m_ref)
    assert np.array_equal(pk.cpu().numpy(), p_ref)
