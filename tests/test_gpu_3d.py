"""GPU parity of the 3-D activation maps (Appendix D) against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2208_04187_amd as pkg
from tests.parity import to_host_array

pytestmark = pytest.mark.gpu

CASES = [
    ((2, 3, 4, 14, 14), 8, 1), ((2, 2, 3, 9, 11), 4, 1), ((2, 2, 3, 35, 35), 4, 1), ((2, 2, 8, 27, 27), 8, 1), ((5, 3, 4, 9, 9), 8, 1),     # 1-bit codes: the units kernels
    ((1, 2, 33, 35, 37), 16, 1), ((3, 4, 2, 4, 6), 8, 1), ((4, 9, 3, 3, 3), 8, 1),     # and the general, one-block and lane kernels
    ((2, 3, 16, 28, 28), 8, 1), ((2, 3, 4, 28, 28), 8, 1), ((1, 2, 20, 44, 48), 8, 1), ((1, 2, 9, 36, 40), 8, 1),   # and the register kernel
    # shape (N, C, D, H, W), B, b                 what it exercises
    ((2, 3, 8, 8, 8), 4, 2),                      # cubes of 4: LDS kernel, vector rows
    ((3, 5, 16, 16, 16), 8, 2),                   # 4096-element planes, several per chunk
    ((2, 3, 5, 9, 13), 4, 2),                     # every extent ragged, odd plane size
    ((2, 2, 6, 10, 7), 3, 4),
    ((5, 7, 4, 12, 20), 8, 4),                    # depth shorter than the block
    ((2, 3, 12, 4, 20), 8, 8),                    # rows shorter than the block
    ((3, 2, 10, 14, 14), 4, 8),
    ((2, 3, 9, 9, 9), 2, 2),                      # 125 blocks per plane
    ((2, 2, 7, 6, 5), 1, 4),                      # B = 1
    ((2, 3, 16, 28, 28), 8, 2),                   # 12544-element planes: register kernel, four wavefronts
    ((2, 3, 4, 28, 28), 8, 4),                    # 3136 elements: register kernel, one wavefront, depth shorter than the block
    ((2, 2, 20, 44, 48), 8, 2),                   # 42240 elements: 1024 threads, ragged blocks in depth and rows
    ((1, 2, 9, 36, 40), 8, 8),                    # ragged everywhere, 8-bit codes
    ((1, 2, 16, 56, 56), 8, 2),                   # plane beyond LDS: workgroup per plane
    ((1, 3, 20, 30, 34), 12, 4),                  # same, ragged, B = 12
    ((1, 2, 40, 40, 40), 8, 8),                   # codes of a plane beyond the staged decompress: stream kernel (fp32), scalar kernel (bf16)
    ((1, 2, 41, 41, 41), 8, 8),                   # the same with odd extents: scalar kernel
    ((1, 2, 33, 35, 37), 16, 2),                  # odd extents beyond LDS: the scalar workgroup-per-plane kernel
    ((2, 3, 18, 44, 48), 8, 4),                   # ragged blocks in depth and rows, workgroup-per-plane kernel
    ((1, 2, 24, 40, 64), 16, 2),
    ((4, 9, 3, 3, 3), 8, 2),                      # one block, odd element count: lane kernels
    ((3, 4, 2, 4, 6), 8, 4),                      # one block, even element count
    ((2, 3, 7, 1, 30), 8, 2),                     # H = 1: a D x W map
    ((2, 3, 7, 30, 1), 8, 2),                     # W = 1: a D x H map
    ((2, 3, 1, 28, 28), 8, 2),                    # D = 1: the 2-D call
    ((70, 9, 4, 4, 4), 4, 2),                     # 630 small planes, ragged last chunk
    ((2, 3, 4, 14, 14), 8, 2),                    # 784 elements, rows of 14: four consecutive elements per lane step
    ((2, 2, 3, 35, 35), 4, 4),                    # odd rows, 3675 elements (odd: 2-byte planes start mid-dword)
    ((2, 2, 8, 27, 27), 8, 2),                    # 5832 elements, four wavefronts per plane
    ((2, 3, 6, 10, 11), 5, 8),                    # blocks of 5: 2 x 2 x 3 of them, ragged in every direction
    ((5, 3, 4, 9, 9), 8, 2),                      # 324 elements: 16 lanes per plane
    ((3, 2, 5, 7, 7), 4, 2),                      # 245 elements: the chunk kernels
]


@pytest.mark.parametrize("shape,B,b", CASES)
@pytest.mark.parametrize("mode", ["f32", "bf16", "c16"])
def test_volumes_match_oracle(shape, B, b, mode):
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    c16 = mode == "c16"
    dt = oracle.F32_C16 if c16 else (oracle.BF16 if mode == "bf16" else oracle.F32)
    g = torch.Generator().manual_seed(9000 + sum(shape) + 17 * B + b)
    x = torch.relu(torch.randn(shape, generator=g) * 1.5 + 0.2).to(dtype)
    x[0, 0] = -2.25                                                   # constant plane: degenerate scale
    xh, _ = to_host_array(x)
    seed = 0x3D3D3D3D00 + B
    ref = oracle.compress(xh, B, b, seed, dt, threads=16)
    need = pkg.division_packed_bytes_3d(*shape, B, b, dtype, c16)
    assert need == ref.size
    pk = torch.full((need,), 0xA5, dtype=torch.uint8, device="cuda:0")
    pkg.division_compress_3d(x.to("cuda:0"), B, b, seed, packed=pk, c16=c16)
    y = pkg.division_decompress_3d(pk, shape, B, b, dtype, c16=c16)
    torch.cuda.synchronize()
    assert np.array_equal(pk.cpu().numpy(), ref)
    yh, _ = to_host_array(y.cpu())
    assert np.array_equal(yh, oracle.decompress(ref, shape, B, b, dt, threads=16))


def test_volume_kernels_cover_what_the_cases_claim():
    kn = pkg.division_kernel_name_3d
    assert kn(0, (3, 5, 16, 16, 16), 8, 2) == "compress_regs_3d<float, 2, 8, 4>"
    assert kn(0, (2, 3, 4, 28, 28), 8, 2) == "compress_regs_3d<float, 2, 8, 1>"
    assert kn(0, (1, 2, 16, 56, 56), 8, 2) == "compress_regs_3d<float, 2, 8, 16>"
    assert kn(0, (1, 2, 16, 56, 56), 8, 2, torch.bfloat16) == "compress_regs_3d<bf16_t, 2, 8, 16>"
    assert kn(0, (2, 3, 5, 9, 13), 4, 2) == "compress_units<float, 2, 1>"
    assert kn(0, (2, 2, 8, 27, 27), 8, 2) == "compress_units<float, 2, 4>"
    assert kn(0, (5, 3, 4, 9, 9), 8, 2) == "compress_units<float, 2, 0>"
    assert kn(0, (3, 2, 5, 7, 7), 4, 2) == "compress_rows_3d<float, 2>"
    assert kn(0, (1, 2, 24, 40, 64), 16, 2) == "compress_plane_3d<float, 2>"
    assert kn(0, (1, 2, 33, 35, 37), 16, 2) == "compress_any_3d<float, 2>"
    assert kn(1, (3, 5, 16, 16, 16), 8, 2) == "decompress_stream_3d<float, 2>"
    assert kn(1, (3, 5, 16, 16, 16), 8, 2, torch.bfloat16) == "decompress_rowvec_3d<bf16_t, 2>"
    assert kn(1, (2, 3, 5, 9, 13), 4, 2) == "decompress_stream_any_3d<float, 2>"
    assert kn(1, (2, 3, 5, 9, 13), 4, 2, torch.bfloat16) == "decompress_units<bf16_t, 2, 1>"
    assert kn(1, (2, 2, 3, 35, 35), 4, 4, torch.bfloat16) == "decompress_units<bf16_t, 4, 2>"
    assert kn(1, (3, 2, 5, 7, 7), 4, 2) == "decompress_stream_any_3d<float, 2>"
    assert kn(1, (3, 2, 5, 7, 7), 4, 2, torch.bfloat16) == "decompress_words_3d<bf16_t, 2>"
    assert kn(1, (2, 2, 6, 10, 7), 3, 4) == "decompress_words_3d<float, 4>"
    assert kn(1, (1, 2, 40, 40, 40), 8, 8) == "decompress_stream_3d<float, 8>"
    assert kn(1, (1, 2, 41, 41, 41), 8, 8) == "decompress_scalar_3d<float, 8>"
    assert kn(0, (4, 9, 3, 3, 3), 8, 2) == "compress_lane<float, 2>"
    assert kn(0, (2, 3, 7, 1, 30), 8, 2) == pkg.division_kernel_name(0, (2, 3, 7, 30), 8, 2)
    assert kn(0, (2, 3, 1, 28, 28), 8, 2) == pkg.division_kernel_name(0, (2, 3, 28, 28), 8, 2)


def test_volume_with_unit_depth_equals_the_2d_call_and_runs_on_a_side_stream():
    x = torch.relu(torch.randn((3, 4, 1, 28, 28), generator=torch.Generator().manual_seed(1))).to("cuda:0")
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        a = pkg.division_compress_3d(x, 8, 2, 77, stream=st)
    st.synchronize()
    b2 = pkg.division_compress(x[:, :, 0].contiguous(), 8, 2, 77)
    torch.cuda.synchronize()
    assert torch.equal(a, b2)


def test_volume_error_codes():
    x = torch.zeros((2, 2, 4, 4, 4), device="cuda:0")
    need = pkg.division_packed_bytes_3d(2, 2, 4, 4, 4, 4, 2)
    small = torch.empty(need - 16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(pkg.DivisionError) as e:
        pkg.division_compress_3d(x, 4, 2, 0, packed=small)
    assert e.value.code == 2                                            # DIVISION_ESIZE
    assert pkg.division_packed_bytes_3d(2, 2, 0, 4, 4, 4, 2) == 0
    assert pkg.division_packed_bytes_3d(2, 2, 4, 4, 4, 4, 3) == 0
    with pytest.raises(ValueError):
        pkg.division_compress_3d(x[0], 4, 2, 0)
    pk = pkg.division_compress_3d(x, 4, 2, 0)
    with pytest.raises(pkg.DivisionError):
        pkg.division_decompress_3d(pk[:-16], (2, 2, 4, 4, 4), 4, 2)
    torch.cuda.synchronize()


@pytest.mark.parametrize("shape,B,b", [((8, 64, 16, 56, 56), 8, 2), ((32, 128, 8, 28, 28), 8, 2), ((4, 16, 16, 112, 112), 8, 4)])
def test_full_size_volumes_match_oracle(shape, B, b):
    """Shapes of a 3-D ResNet-18 on 16 x 112 x 112 clips (workgroup-per-plane and chunked kernels), whole tensor."""
    g = torch.Generator().manual_seed(sum(shape))
    x = torch.relu(torch.randn(shape, generator=g))
    seed = 0xF00D + B
    ref = oracle.compress(x.numpy(), B, b, seed, threads=16)
    pk = pkg.division_compress_3d(x.to("cuda:0"), B, b, seed)
    y = pkg.division_decompress_3d(pk, shape, B, b)
    torch.cuda.synchronize()
    assert np.array_equal(pk.cpu().numpy(), ref)
    assert np.array_equal(y.cpu().numpy(), oracle.decompress(ref, shape, B, b, threads=16))


def _volume_sweep(n, seed0):
    rng = np.random.default_rng(seed0)
    cases = []
    for _ in range(n):
        D = int(rng.choice([1, 2, 3, 4, 5, 8, 9, 16, 17]))
        H = int(rng.integers(1, 41))
        W = int(rng.choice([H, int(rng.integers(1, 61)), 4 * int(rng.integers(1, 16)), 8 * int(rng.integers(1, 9))]))
        B = int(rng.choice([1, 2, 3, 4, 4, 5, 8, 8, 8, 12, 16, 18, 64]))
        b = int(rng.choice([2, 2, 4, 8]))
        N, C = int(rng.integers(1, 5)), int(rng.integers(1, 9))
        if D * H * W <= 256 and rng.random() < 0.5:
            N, C = int(rng.integers(10, 60)), int(rng.integers(3, 9))
        mode = str(rng.choice(["f32", "f32", "bf16", "c16"]))
        cases.append(((N, C, D, H, W), B, b, mode, int(rng.integers(0, 2 ** 63))))
    return cases


@pytest.mark.parametrize("chunk", range(4))
def test_seeded_sweep_of_volumes(chunk):
    """160 pseudo-random (shape, B, b, format, seed) combinations of 3-D maps, 40 per test."""
    for shape, B, b, mode, seed in _volume_sweep(160, 20260117)[40 * chunk:40 * (chunk + 1)]:
        dtype = torch.bfloat16 if mode == "bf16" else torch.float32
        c16 = mode == "c16"
        dt = oracle.F32_C16 if c16 else (oracle.BF16 if mode == "bf16" else oracle.F32)
        g = torch.Generator().manual_seed(seed % 100003)
        x = torch.relu(torch.randn(shape, generator=g) + 0.3).to(dtype)
        xh, _ = to_host_array(x)
        ref = oracle.compress(xh, B, b, seed, dt)
        need = pkg.division_packed_bytes_3d(*shape, B, b, dtype, c16)
        pk = torch.full((need,), 0x5A, dtype=torch.uint8, device="cuda:0")
        pkg.division_compress_3d(x.to("cuda:0"), B, b, seed, packed=pk, c16=c16)
        y = pkg.division_decompress_3d(pk, shape, B, b, dtype, c16=c16)
        torch.cuda.synchronize()
        tag = f"shape={shape} B={B} b={b} mode={mode} seed={seed} kernel={pkg.division_kernel_name_3d(0, shape, B, b, dtype, c16=c16)}"
        assert np.array_equal(pk.cpu().numpy(), ref), tag
        yh, _ = to_host_array(y.cpu())
        assert np.array_equal(yh, oracle.decompress(ref, shape, B, b, dt)), tag


# values at the edges of binary32 (zero, constant, subnormal, overflowing and signed-zero planes) under the volume kernels
@pytest.mark.parametrize("shape,B", [((1, 12, 16, 16, 16), 8), ((1, 12, 4, 28, 28), 8), ((1, 12, 16, 56, 56), 8),
                                      ((2, 6, 5, 9, 13), 4), ((2, 6, 8, 27, 27), 8), ((3, 4, 4, 9, 9), 8), ((3, 4, 5, 7, 7), 4),
                                      ((1, 12, 24, 40, 64), 16), ((1, 12, 33, 35, 37), 16), ((4, 3, 3, 3, 3), 8)])
@pytest.mark.parametrize("mode,b", [("f32", 2), ("bf16", 4), ("c16", 8)])
def test_volumes_with_values_at_the_edges_of_binary32(shape, B, mode, b):
    from tests.test_gpu_parity import _special_planes
    dtype = torch.bfloat16 if mode == "bf16" else torch.float32
    c16 = mode == "c16"
    dt = oracle.F32_C16 if c16 else (oracle.BF16 if mode == "bf16" else oracle.F32)
    N, C, D, H, W = shape
    x = _special_planes((N, C, D * H, W), 57 + B).view(shape).to(dtype)
    xh, _ = to_host_array(x)
    ref = oracle.compress(xh, B, b, 4048, dt, threads=16)
    pk = pkg.division_compress_3d(x.to("cuda:0"), B, b, 4048, c16=c16)
    y = pkg.division_decompress_3d(pk, shape, B, b, dtype, c16=c16)
    torch.cuda.synchronize()
    assert np.array_equal(pk.cpu().numpy(), ref), pkg.division_kernel_name_3d(0, shape, B, b, dtype, c16=c16)
    yh, _ = to_host_array(y.cpu())
    assert np.array_equal(yh, oracle.decompress(ref, shape, B, b, dt, threads=16), equal_nan=mode != "bf16")
