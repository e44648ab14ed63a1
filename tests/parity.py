"""Shared helpers of the GPU parity tests: run the HIP path and the CPU oracle
on the same host array and compare them to the stated bar.

Bar (from the benchmark spec):
  * packed HFC codes bit-exact, except a mismatch rate <= 1e-6 of +-1 flips
    whose pre-round value t + r/2^16 lies within 1e-6 * max(1, t) of an integer;
  * LFC and (delta, Delta) within 1e-5 relative (fp32) / 1e-2 (bf16);
  * decompression is a pure function of the packed buffer, so the GPU's
    reconstruction must equal the oracle's reconstruction OF THE GPU'S PACKED
    BUFFER bit for bit; against the oracle's own round trip it may differ only
    where a code legitimately flipped or where the LFC / scale differ in the
    last bits (tolerance rtol * (|xhat| + plane magnitude)).
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2208_04187_amd as pkg


def to_host_array(x: torch.Tensor):
    """float32 tensor -> float32 ndarray; bfloat16 tensor -> uint16 bit patterns."""
    if x.dtype == torch.bfloat16:
        return x.contiguous().view(torch.int16).numpy().view(np.uint16), oracle.BF16
    return x.contiguous().numpy(), oracle.F32


def gpu_roundtrip(x: torch.Tensor, B: int, b: int, seed: int, prefill: int | None = 0xFF):
    xd = x.to("cuda:0")
    N, C, H, W = x.shape
    need = pkg.division_packed_bytes(N, C, H, W, B, b, x.dtype)
    packed = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    if prefill is not None:
        packed.fill_(prefill)
    pkg.division_compress(xd, B, b, seed, packed=packed)
    xhat = pkg.division_decompress(packed, tuple(x.shape), B, b, x.dtype)
    torch.cuda.synchronize()
    return packed.cpu().numpy(), xhat.cpu()


def check_against_oracle(x: torch.Tensor, B: int, b: int, seed: int, threads: int = 1,
                         require_exact: bool = False) -> dict:
    """Runs both sides; asserts the bar; returns statistics."""
    xh, dt = to_host_array(x)
    shape = tuple(x.shape)
    N, C, H, W = shape
    HW = H * W
    gp, gx = gpu_roundtrip(x, B, b, seed)
    rp = oracle.compress(xh, B, b, seed, dt, threads=threads)
    assert gp.size == rp.size == oracle.packed_bytes(N, C, H, W, B, b, dt)
    gxh, _ = to_host_array(gx)

    # decompression of the GPU's own packed buffer: bit-exact
    assert np.array_equal(gxh, oracle.decompress(gp, shape, B, b, dt, threads=threads)), \
        "GPU decompress differs from the oracle's decompress of the same packed buffer"

    stats = {"elements": x.numel(), "exact": bool(np.array_equal(gp, rp)), "flips": 0}
    if stats["exact"]:
        return stats
    assert not require_exact, "packed buffer differs from the oracle"

    g, r = oracle.split_packed(gp, shape, B, b, dt), oracle.split_packed(rp, shape, B, b, dt)
    rtol = 1e-2 if dt == oracle.BF16 else 1e-5
    lg = oracle.bf16_to_f32(g["lfc"]) if dt == oracle.BF16 else g["lfc"]
    lr = oracle.bf16_to_f32(r["lfc"]) if dt == oracle.BF16 else r["lfc"]
    scale = np.abs(xh if dt == oracle.F32 else oracle.bf16_to_f32(xh)).reshape(N * C, -1).max(1)
    assert np.all(np.abs(lg - lr) <= rtol * (np.abs(lr) + 1e-30) + 1e-6 * rtol * scale[:, None, None]), "LFC out of tolerance"
    assert np.all(np.abs(g["meta"] - r["meta"]) <= rtol * np.abs(r["meta"]) + 4e-7 * scale[:, None]), "meta out of tolerance"

    qg, qr = oracle.unpack_codes(g["codes"], HW, b), oracle.unpack_codes(r["codes"], HW, b)
    diff = qg.astype(np.int16) - qr.astype(np.int16)
    bad = np.nonzero(diff)
    stats["flips"] = int(bad[0].size)
    assert stats["flips"] <= 1e-6 * x.numel() + 0.5, f"{stats['flips']} code mismatches in {x.numel()} elements"
    # pad bits of the last word of every plane are zero on both sides
    if bad[0].size:
        assert np.all(np.abs(diff[bad]) == 1), "a code differs by more than one step"
        _, dbg = oracle.compress(xh, B, b, seed, dt, threads=threads, debug=True)
        t = dbg["t"].reshape(N * C, HW)[bad].astype(np.float64)
        s = t + dbg["r"].reshape(N * C, HW)[bad].astype(np.float64) / 65536.0
        dist = np.abs(s - np.round(s))
        assert np.all(dist <= 1e-6 * np.maximum(1.0, t)), "a flipped code was not at a rounding boundary"
    return stats
