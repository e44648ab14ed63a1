"""A bounded, seeded slice of random shapes through the HIP library against the CPU oracle, bit for bit:
1-D, 2-D and 3-D maps, block sizes 1..128, code widths 2 / 4 / 8, the three element / cache types, with
planes at the edges of binary32 planted in a third of the cases.  Stops at the first mismatch and names
the case.  (Sec. 4.1 / 4.2, Appendix D; the bar is the one of tests/parity.py with no flips allowed.)
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2208_04187_amd as pkg

pytestmark = pytest.mark.gpu


def _host(x):
    return x.contiguous().view(torch.int16).numpy().view(np.uint16) if x.dtype == torch.bfloat16 else x.numpy()


def _draw_case(rng, one_bit=False):
    three = rng.random() < 0.3
    kind = rng.integers(0, 6)
    if kind == 0:
        H = W = int(rng.choice([4, 7, 8, 13, 14, 16, 17, 27, 28, 32, 35, 55, 56, 64, 73, 112]))
    elif kind == 1:
        H, W = int(rng.integers(1, 80)), int(rng.integers(1, 80))
    elif kind == 2:
        H, W = 1, int(rng.choice([24, 64, 96, 128, 196, 200, 384, 768, 1000, 1024, 3072, 4096]))
    elif kind == 3:
        H, W = int(rng.integers(1, 40)), 4 * int(rng.integers(1, 40))
    elif kind == 4:
        H, W = int(rng.integers(100, 320)), int(rng.integers(100, 320))
    else:
        H, W = 8 * int(rng.integers(1, 20)), 8 * int(rng.integers(1, 20))
    D = int(rng.choice([2, 3, 4, 8, 16])) if three else 1
    if three and D * H * W > 300000:
        H, W = H // 4 + 1, W // 4 + 1
    B = int(rng.choice([1, 2, 3, 4, 4, 4, 5, 6, 8, 8, 8, 8, 12, 16, 18, 32, 64, 128]))
    b = int(rng.choice([1, 1, 2, 4, 8])) if one_bit else int(rng.choice([2, 2, 4, 8]))
    maxpl = max(1, 600000 // (D * H * W))
    P = int(rng.integers(1, min(maxpl, 400) + 1))
    C = int(rng.integers(1, P + 1))
    N = max(1, P // C)
    mode = str(rng.choice(["f32", "f32", "bf16", "c16"]))
    shape = (N, C, D, H, W) if three else (N, C, H, W)
    g = torch.Generator().manual_seed(int(rng.integers(0, 2 ** 31)))
    x = torch.randn(shape, generator=g) * float(rng.choice([0.01, 1.0, 300.0]))
    if rng.random() < 0.6:
        x = torch.relu(x)
    if rng.random() < 0.3:
        # zeros of both signs, subnormals, tiny and overflowing ranges, an outlier, a constant
        xp = x.view(N * C, -1)
        for p_ in rng.choice(N * C, size=min(N * C, 4), replace=False):
            r_ = torch.randn(xp.shape[1], generator=g)
            xp[int(p_)] = [torch.zeros_like(r_), -torch.zeros_like(r_), r_ * 1e-41, r_ * 1e-30, r_ * 1e-26,
                           torch.sign(r_) * 1.6e38, torch.where(r_ > 2, 1e30, 1.0) * r_, torch.full_like(r_, -2.5),
                           torch.where(r_ > 0, 0.0, -0.0)][int(rng.integers(0, 9))]
    seed = int(rng.integers(0, 2 ** 63))
    return three, shape, B, b, mode, x, seed


# (the third slice draws 1-bit codes in two cases of five)
@pytest.mark.parametrize("rng_seed,cases", [(21, 150), (22, 150), (23, 200)])
def test_random_shapes_bit_exact(rng_seed, cases):
    rng = np.random.default_rng(rng_seed)
    kernels = set()
    for k in range(cases):
        three, shape, B, b, mode, x, seed = _draw_case(rng, one_bit=rng_seed == 23)
        dtype = torch.bfloat16 if mode == "bf16" else torch.float32
        c16 = mode == "c16"
        dt = oracle.F32_C16 if c16 else (oracle.BF16 if mode == "bf16" else oracle.F32)
        x = x.to(dtype)
        what = f"case {k} of rng {rng_seed}: shape {shape} B={B} b={b} {mode} seed={seed}"
        ref = oracle.compress(_host(x), B, b, seed, dt, threads=8)
        xd = x.to("cuda:0")
        if three:
            names = (pkg.division_kernel_name_3d(0, shape, B, b, dtype, c16=c16), pkg.division_kernel_name_3d(1, shape, B, b, dtype, c16=c16))
            pk = pkg.division_compress_3d(xd, B, b, seed, c16=c16)
            y = pkg.division_decompress_3d(pk, shape, B, b, dtype, c16=c16)
        else:
            names = (pkg.division_kernel_name(0, shape, B, b, dtype, c16=c16), pkg.division_kernel_name(1, shape, B, b, dtype, c16=c16))
            pk = pkg.division_compress(xd, B, b, seed, c16=c16)
            y = pkg.division_decompress(pk, shape, B, b, dtype, c16=c16)
        torch.cuda.synchronize()
        assert np.array_equal(pk.cpu().numpy(), ref), f"packed buffer differs ({names[0]}); {what}"
        assert np.array_equal(_host(y.cpu()), oracle.decompress(ref, shape, B, b, dt, threads=8), equal_nan=mode != "bf16"), f"x-hat differs ({names[1]}); {what}"
        kernels.update(n.split("<")[0] for n in names)
    assert len(kernels) >= 12, sorted(kernels)          # the slice reaches most kernel families
