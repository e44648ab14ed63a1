"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and its host-only entry points agree with
the oracle's byte accounting and reject bad arguments."""
import ctypes
import os
import re

import pytest

import oracle
import paper_2208_04187_amd as pkg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "division.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(division_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert {"division_packed_bytes", "division_compress", "division_decompress",
            "division_packed_layout", "division_abi_version",
            "division_compress_batch", "division_decompress_batch"} <= set(names)
    L = pkg.lib()
    for n in names:
        assert hasattr(L, n), n
    assert L.division_abi_version() == 1


SHAPES = [(2, 16, 32, 32, 8, 2), (64, 256, 56, 56, 8, 2), (64, 2048, 7, 7, 8, 2), (32, 96, 55, 55, 4, 4),
          (128, 512, 4, 4, 4, 2), (1, 1, 1, 1, 1, 2), (3, 5, 13, 29, 5, 4), (2, 2, 300, 300, 64, 2)]


@pytest.mark.parametrize("dt", [0, 1])
def test_packed_bytes_and_layout_match_oracle(dt):
    import torch
    tdt = torch.float32 if dt == 0 else torch.bfloat16
    for s in SHAPES:
        assert pkg.division_packed_bytes(*s, dtype=tdt) == oracle.packed_bytes(*s, dt)
        assert pkg.division_packed_layout(*s, dtype=tdt) == oracle.packed_layout(*s, dt)


def test_config_sizes_and_ratios():
    # sizes of the benchmark configurations (fp32 LFC, 8-byte meta)
    assert pkg.division_packed_bytes(2, 16, 32, 32, 8, 2) == 10496
    from synthetic_inputs import config
    _, specs = config(2)
    inp = sum(4 * s.shape[0] * s.shape[1] * s.shape[2] * s.shape[3] for s in specs)
    out = sum(pkg.division_packed_bytes(*s.shape, s.B, s.b) for s in specs)
    assert inp == 1618477056
    assert 11.4 < inp / out < 11.6          # >= 10x activation compression at B=8, b=2


def test_invalid_arguments_are_rejected_on_the_host():
    L = pkg.lib()
    assert L.division_packed_bytes(0, 1, 4, 4, 2, 2, 0) == 0
    assert L.division_packed_bytes(1, 1, 4, 4, 0, 2, 0) == 0
    assert L.division_packed_bytes(1, 1, 4, 4, 2, 3, 0) == 0
    assert L.division_packed_bytes(1, 1, 4, 4, 2, 2, 7) == 0
    assert L.division_packed_bytes(2 ** 20, 2 ** 20, 4, 4, 2, 2, 0) == 0        # too many planes
    buf = ctypes.create_string_buffer(4096)
    addr = ctypes.addressof(buf)
    addr16 = (addr + 15) & ~15
    # all of these return before any HIP call is made
    assert L.division_compress(None, 1, 1, 4, 4, 0, 2, 2, 0, addr16, 4096, None) == 1
    assert L.division_compress(addr16, 1, 1, 4, 4, 0, 2, 5, 0, addr16, 4096, None) == 1
    assert L.division_compress(addr16, 1, 1, 4, 4, 0, 2, 2, 0, addr16 + 1024, 8, None) == 2
    assert L.division_compress(addr16, 1, 1, 4, 4, 0, 2, 2, 0, addr16 + 1025, 2048, None) == 3
    assert L.division_compress(addr16 + 2, 1, 1, 4, 4, 0, 2, 2, 0, addr16 + 1024, 2048, None) == 3
    assert L.division_compress(addr16, 2 ** 20, 2 ** 20, 4, 4, 0, 2, 2, 0, addr16 + 1024, 2048, None) == 4
    assert L.division_decompress(None, 64, 1, 1, 4, 4, 0, 2, 2, addr16, None) == 1
    assert L.division_decompress(addr16, 8, 1, 1, 4, 4, 0, 2, 2, addr16 + 1024, None) == 2
    assert L.division_decompress(addr16 + 4, 2048, 1, 1, 4, 4, 0, 2, 2, addr16 + 1024, None) == 3
    # the batch forms check every item before anything is launched
    vp2 = ctypes.c_void_p * 2
    xs, pk = vp2(addr16, addr16 + 512), vp2(addr16 + 1024, addr16 + 2048)
    sd = (ctypes.c_uint64 * 2)(1, 2)
    assert L.division_compress_batch(0, None, None, None, 1, 1, 4, 4, 0, 2, 2, 2048, None) == 0
    assert L.division_compress_batch(-1, xs, pk, sd, 1, 1, 4, 4, 0, 2, 2, 2048, None) == 1
    assert L.division_compress_batch(2, xs, None, sd, 1, 1, 4, 4, 0, 2, 2, 2048, None) == 1
    assert L.division_compress_batch(2, vp2(addr16, None), pk, sd, 1, 1, 4, 4, 0, 2, 2, 2048, None) == 1
    assert L.division_compress_batch(2, xs, pk, sd, 1, 1, 4, 4, 0, 2, 2, 8, None) == 2
    assert L.division_compress_batch(2, xs, vp2(addr16 + 1024, addr16 + 2049), sd, 1, 1, 4, 4, 0, 2, 2, 1024, None) == 3
    assert L.division_decompress_batch(0, None, None, 64, 1, 1, 4, 4, 0, 2, 2, None) == 0
    assert L.division_decompress_batch(2, pk, None, 64, 1, 1, 4, 4, 0, 2, 2, None) == 1
    assert L.division_decompress_batch(2, pk, xs, 8, 1, 1, 4, 4, 0, 2, 2, None) == 2
    assert L.division_decompress_batch(2, pk, vp2(addr16, addr16 + 2), 1024, 1, 1, 4, 4, 0, 2, 2, None) == 3


def test_descriptor_array_calls_check_every_map_before_any_launch():
    from paper_2208_04187_amd.binding import _MapDesc
    L = pkg.lib()
    buf = ctypes.create_string_buffer(8192)
    a = (ctypes.addressof(buf) + 15) & ~15
    good = dict(x=a, packed=a + 1024, xhat=a + 2048, packed_bytes=1024, N=1, C=1, D=1, H=4, W=4, dt=0, B=2, b=2, seed=3)

    def call(fn, *over):
        descs = (_MapDesc * len(over))(*[_MapDesc(**{**good, **o}) for o in over])
        return fn(len(over), descs, None)

    assert L.division_compress_maps(0, None, None) == 0
    assert L.division_compress_maps(2, None, None) == 1
    assert L.division_compress_maps(-1, None, None) == 1
    # the second map is invalid: nothing is launched (no HIP call is made on this GPU-less host)
    assert call(L.division_compress_maps, {}, {"x": None}) == 1
    assert call(L.division_compress_maps, {}, {"b": 3}) == 1
    assert call(L.division_compress_maps, {}, {"D": 0}) == 1
    assert call(L.division_compress_maps, {}, {"packed_bytes": 16}) == 2
    assert call(L.division_compress_maps, {}, {"packed": a + 1025}) == 3
    assert call(L.division_compress_maps, {}, {"N": 2 ** 20, "C": 2 ** 20}) == 4
    assert call(L.division_decompress_maps, {}, {"xhat": None}) == 1
    assert call(L.division_decompress_maps, {}, {"x": None, "xhat": a + 2050}) == 3
    assert call(L.division_decompress_maps, {}, {"packed_bytes": 8}) == 2
    assert ctypes.sizeof(_MapDesc) == 96          # the C struct: 3 pointers, size_t, 5 x int64, 3 x int (+ pad), uint64


def test_mask_bytes_and_host_side_errors():
    L = pkg.lib()
    for n in (0, 1, 31, 32, 33, 1 << 20, (1 << 31) + 5):
        assert pkg.division_mask_bytes(n) == oracle.mask_bytes(n) == 4 * ((n + 31) // 32)
    assert L.division_mask_bytes(-1) == 0
    buf = ctypes.create_string_buffer(4096)
    a16 = (ctypes.addressof(buf) + 15) & ~15
    # all of these return before any HIP call is made
    assert L.division_relu_forward(None, 8, 0, a16, a16 + 512, 4, None) == 1
    assert L.division_relu_forward(a16, -1, 0, a16, a16 + 512, 4, None) == 1
    assert L.division_relu_forward(a16, 8, 5, a16, a16 + 512, 4, None) == 1
    assert L.division_relu_forward(a16, 64, 0, a16, a16 + 512, 4, None) == 2
    assert L.division_relu_forward(a16 + 2, 8, 0, a16, a16 + 512, 4, None) == 3
    assert L.division_relu_forward(a16, 8, 0, a16, a16 + 513, 4, None) == 3
    assert L.division_relu_forward(a16, (1 << 40) + 1, 0, a16, a16 + 512, 1 << 40, None) == 4
    assert L.division_relu_forward(a16, 0, 0, a16, a16 + 512, 0, None) == 0
    assert L.division_dropout_forward(a16, 8, 1, 0.5, 1, None, a16 + 512, 4, None) == 1
    assert L.division_mask_backward(a16 + 512, 0, a16, 8, 0, a16, None) == 2


def test_layout_of_the_bfloat16_cached_mode_matches_oracle():
    import torch
    for s in SHAPES:
        assert pkg.division_packed_bytes(*s, dtype=torch.float32, c16=True) == oracle.packed_bytes(*s, oracle.F32_C16)
        assert pkg.division_packed_layout(*s, dtype=torch.float32, c16=True) == oracle.packed_layout(*s, oracle.F32_C16)
    with pytest.raises(TypeError):
        pkg.division_packed_bytes(1, 1, 4, 4, 2, 2, dtype=torch.bfloat16, c16=True)
    assert pkg.lib().division_packed_bytes(1, 1, 4, 4, 2, 2, 3) == 0           # unknown dtype code


def test_layout_matches_oracle_over_a_seeded_grid_of_shapes():
    """The two layouts are typed independently (csrc/host.h, oracle/division_oracle.c): 2-D and 3-D maps, every code
    width incl. 1 bit, the three cache formats, block sizes below, at and above the extents."""
    import numpy as np
    import torch
    rng = np.random.default_rng(20220808)
    fmts = [(torch.float32, False, oracle.F32), (torch.bfloat16, False, oracle.BF16), (torch.float32, True, oracle.F32_C16)]
    for _ in range(1500):
        N, C = int(rng.integers(1, 70)), int(rng.integers(1, 300))
        H, W = int(rng.integers(1, 240)), int(rng.integers(1, 240))
        B = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 18, 64, 300]))
        b = int(rng.choice([1, 2, 4, 8]))
        tdt, c16, odt = fmts[int(rng.integers(0, 3))]
        if rng.random() < 0.3:
            D = int(rng.integers(2, 20))
            assert pkg.division_packed_bytes_3d(N, C, D, H, W, B, b, tdt, c16) == oracle.packed_bytes_3d(N, C, D, H, W, B, b, odt)
            assert pkg.division_packed_layout_3d(N, C, D, H, W, B, b, tdt, c16) == oracle.packed_layout_3d(N, C, D, H, W, B, b, odt)
        else:
            assert pkg.division_packed_bytes(N, C, H, W, B, b, tdt, c16) == oracle.packed_bytes(N, C, H, W, B, b, odt)
            assert pkg.division_packed_layout(N, C, H, W, B, b, tdt, c16) == oracle.packed_layout(N, C, H, W, B, b, odt)


def test_the_planner_names_a_kernel_for_every_shape_of_a_seeded_grid():
    """Host-side only: for every valid shape, code width, format and pointer alignment the planner answers with a
    kernel of a known family whose template arguments carry the code width asked for."""
    import numpy as np
    import torch
    rng = np.random.default_rng(4187)
    comp = {"compress_regs", "compress_regs_3d", "compress_lane", "compress_line", "compress_strip", "compress_rowstrip",
            "compress_items", "compress_units", "compress_wave", "compress_tile", "compress_one", "compress_rows",
            "compress_rows_3d", "compress_plane", "compress_plane_3d", "compress_any", "compress_any_3d"}
    dec = {"decompress_stream", "decompress_stream_3d", "decompress_stream_any", "decompress_stream_any_3d",
           "decompress_stream_one", "decompress_rowvec", "decompress_rowvec_3d", "decompress_table", "decompress_units",
           "decompress_words", "decompress_words_3d", "decompress_flat", "decompress_flat_3d", "decompress_lane",
           "decompress_scalar", "decompress_scalar_3d"}
    seen = set()
    for _ in range(4000):
        N, C = int(rng.integers(1, 40)), int(rng.integers(1, 100))
        H, W = int(rng.integers(1, 200)), int(rng.integers(1, 200))
        if rng.random() < 0.3:
            H = W = int(rng.choice([4, 7, 8, 13, 14, 16, 17, 27, 28, 32, 35, 55, 56, 73, 112, 147]))
        B = int(rng.choice([1, 2, 3, 4, 8, 8, 12, 16, 18, 64]))
        b = int(rng.choice([1, 2, 4, 8]))
        tdt, c16 = [(torch.float32, False), (torch.bfloat16, False), (torch.float32, True)][int(rng.integers(0, 3))]
        ptr = int(rng.choice([0, 256, 260, 258])) if tdt == torch.bfloat16 else int(rng.choice([0, 256, 260]))
        three = rng.random() < 0.25
        shape = (N, C, int(rng.integers(2, 12)), H, W) if three else (N, C, H, W)
        kn = pkg.division_kernel_name_3d if three else pkg.division_kernel_name
        for direction, families in ((0, comp), (1, dec)):
            name = kn(direction, shape, B, b, tdt, data_ptr=ptr, c16=c16)
            family, args = name.split("<", 1)
            assert family in families, name
            assert args.split(", ")[1].rstrip(">") == str(b), name
            seen.add(family)
    assert len(seen) >= 28, sorted(seen)


# which kernel the host picks for a shape (a host-side decision: no GPU needed to ask)
DISPATCH = [
    # shape, B, b, compress kernel, decompress kernel (fp32)
    ((64, 256, 56, 56), 8, 2, "compress_regs<float, 2, 8, 1>", "decompress_stream<float, 2>"),
    # 1-bit codes: the ResNet-50 shapes in the fast kernels, the rest in the general ones
    ((64, 256, 56, 56), 8, 1, "compress_regs<float, 1, 8, 1>", "decompress_stream<float, 1>"),
    ((64, 64, 112, 112), 8, 1, "compress_regs<float, 1, 8, 4>", "decompress_stream<float, 1>"),
    ((64, 512, 28, 28), 8, 1, "compress_strip<float, 1, 28, 8>", "decompress_stream<float, 1>"),
    ((64, 1024, 14, 14), 8, 1, "compress_strip<float, 1, 14, 8>", "decompress_table<float, 1>"),
    ((64, 2048, 7, 7), 8, 1, "compress_lane<float, 1>", "decompress_lane<float, 1>"),
    ((256, 96, 55, 55), 8, 1, "compress_rowstrip<float, 1, 55, 8>", "decompress_stream_any<float, 1>"),
    ((128, 768, 17, 17), 8, 1, "compress_rowstrip<float, 1, 17, 8>", "decompress_stream_any<float, 1>"),
    ((256, 256, 8, 8), 4, 1, "compress_items<float, 1, 4, 4, 4>", "decompress_stream<float, 1>"),
    ((64, 64, 147, 147), 8, 1, "compress_tile<float, 1, 8, 1, 256>", "decompress_stream_any<float, 1>"),
    ((64, 64, 147, 147), 18, 1, "compress_any<float, 1>", "decompress_stream_any<float, 1>"),
    ((64, 96, 64, 64), 8, 1, "compress_tile<float, 1, 8, 4, 256>", "decompress_stream<float, 1>"),
    ((256, 128, 1, 768), 8, 1, "compress_line<float, 1, 6, 1>", "decompress_stream<float, 1>"),
    ((64, 256, 56, 56), 64, 1, "compress_one<float, 1, 13>", "decompress_stream<float, 1>"),
    ((64, 512, 28, 28), 3, 1, "compress_any<float, 1>", "decompress_table<float, 1>"),
    ((64, 64, 112, 112), 8, 2, "compress_regs<float, 2, 8, 4>", "decompress_stream<float, 2>"),
    ((2, 3, 224, 224), 8, 2, "compress_regs<float, 2, 8, 16>", "decompress_stream<float, 2>"),
    ((64, 512, 28, 28), 8, 2, "compress_strip<float, 2, 28, 8>", "decompress_stream<float, 2>"),
    ((64, 1024, 14, 14), 8, 2, "compress_strip<float, 2, 14, 8>", "decompress_table<float, 2>"),
    ((4, 8, 20, 28), 8, 4, "compress_strip<float, 4, 28, 8>", "decompress_stream<float, 4>"),
    ((256, 64, 32, 32), 12, 2, "compress_strip<float, 2, 32, 12>", "decompress_stream<float, 2>"),     # the block-size sweep on CIFAR maps
    ((256, 64, 32, 32), 18, 2, "compress_strip<float, 2, 32, 18>", "decompress_table<float, 2>"),
    ((256, 128, 16, 16), 12, 2, "compress_strip<float, 2, 16, 12>", "decompress_stream<float, 2>"),
    ((64, 512, 28, 28), 18, 2, "compress_strip<float, 2, 28, 18>", "decompress_table<float, 2>"),
    ((64, 1024, 14, 14), 12, 2, "compress_strip<float, 2, 14, 12>", "decompress_table<float, 2>"),
    ((4, 8, 28, 28), 4, 2, "compress_items<float, 2, 4, 4, 4>", "decompress_stream<float, 2>"),
    ((4, 8, 15, 14), 8, 2, "compress_items<float, 2, 8, 2, 8>", "decompress_stream_any<float, 2>"),
    ((64, 2048, 7, 7), 8, 2, "compress_lane<float, 2>", "decompress_lane<float, 2>"),
    ((128, 64, 32, 32), 4, 2, "compress_strip<float, 2, 32, 4>", "decompress_stream<float, 2>"),
    ((128, 128, 16, 16), 4, 2, "compress_strip<float, 2, 16, 4>", "decompress_stream<float, 2>"),
    ((128, 256, 8, 8), 4, 2, "compress_items<float, 2, 4, 4, 4>", "decompress_stream<float, 2>"),
    ((64, 256, 56, 56), 12, 2, "compress_regs<float, 2, 0, 1>", "decompress_stream<float, 2>"),
    ((64, 256, 56, 56), 64, 2, "compress_one<float, 2, 13>", "decompress_stream<float, 2>"),
    ((64, 256, 56, 56), 18, 4, "compress_units<float, 4, 2>", "decompress_table<float, 4>"),
    ((32, 96, 55, 55), 4, 4, "compress_rowstrip<float, 4, 55, 4>", "decompress_stream_any<float, 4>"),
    ((8, 8, 27, 27), 8, 2, "compress_rowstrip<float, 2, 27, 8>", "decompress_stream_any<float, 2>"),
    ((8, 8, 17, 17), 8, 2, "compress_rowstrip<float, 2, 17, 8>", "decompress_stream_any<float, 2>"),
    ((8, 8, 13, 13), 8, 2, "compress_rowstrip<float, 2, 13, 8>", "decompress_stream_any<float, 2>"),
    ((8, 8, 27, 27), 4, 2, "compress_rowstrip<float, 2, 27, 4>", "decompress_stream_any<float, 2>"),
    ((8, 8, 29, 29), 4, 2, "compress_units<float, 2, 1>", "decompress_stream_any<float, 2>"),
    ((8, 8, 19, 19), 8, 2, "compress_units<float, 2, 0>", "decompress_stream_any<float, 2>"),
    ((8, 8, 11, 11), 8, 2, "compress_wave<float, 2, 8, 1>", "decompress_stream_any<float, 2>"),
    ((8, 8, 35, 35), 8, 2, "compress_rowstrip<float, 2, 35, 8>", "decompress_stream_any<float, 2>"),
    ((8, 8, 73, 73), 8, 2, "compress_units<float, 2, 4>", "decompress_stream_any<float, 2>"),
    ((4, 4, 147, 147), 8, 2, "compress_units<float, 2, 16>", "decompress_stream_any<float, 2>"),
    ((4, 4, 30, 30), 4, 2, "compress_wave<float, 2, 4, 2>", "decompress_table<float, 2>"),
    ((2, 2, 1, 768), 8, 4, "compress_line<float, 4, 6, 1>", "decompress_stream<float, 4>"),
    ((5, 33, 14, 14), 12, 4, "compress_strip<float, 4, 14, 12>", "decompress_table<float, 4>"),
    ((5, 33, 24, 24), 18, 4, "compress_rows<float, 4>", "decompress_table<float, 4>"),
    ((1, 1, 300, 300), 18, 2, "compress_any<float, 2>", "decompress_scalar<float, 2>"),
]


@pytest.mark.parametrize("shape,B,b,comp,dec", DISPATCH)
def test_kernel_choice_per_shape(shape, B, b, comp, dec):
    assert pkg.division_kernel_name(0, shape, B, b) == comp
    assert pkg.division_kernel_name(1, shape, B, b) == dec


def test_kernel_choice_for_3d_maps_and_2_byte_elements():
    import torch
    assert pkg.division_kernel_name_3d(0, (2, 4, 16, 56, 56), 8, 2) == "compress_regs_3d<float, 2, 8, 16>"
    assert pkg.division_kernel_name_3d(1, (2, 4, 16, 56, 56), 8, 2) == "decompress_stream_3d<float, 2>"
    assert pkg.division_kernel_name(0, (8, 8, 55, 55), 8, 2, torch.bfloat16) == "compress_rowstrip<bf16_t, 2, 55, 8>"
    assert pkg.division_kernel_name(0, (8, 8, 55, 55), 18, 2, torch.bfloat16) == "compress_units<bf16_t, 2, 2>"
    assert pkg.division_kernel_name(1, (8, 8, 55, 55), 8, 2, torch.bfloat16) == "decompress_units<bf16_t, 2, 2>"
    assert pkg.division_kernel_name(0, (8, 8, 56, 56), 8, 2, torch.float32, c16=True) == "compress_regs<f32c16_t, 2, 8, 1>"
