#!/usr/bin/env python3
"""Benchmark of the DIVISION activation codec on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic
activations: every tensor of the workload is compressed (forward order), then
every tensor is decompressed (reverse order, as the backward pass of
Algorithm 1 does).  Inputs are resident in HBM before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config IDX]

Prints ONE JSON line.  `value` is the algorithmic throughput
2 * (input_bytes + packed_bytes) / step_time in GB/s (bytes the method must
move: one read of x and one write of the packed tuple in compress, the reverse
in decompress); `activation_GB_s` counts the activation bytes alone.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth

TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_resnet50_set_hbm_traffic.md")


def recorded_traffic(kernel: str, launches_per_step: int, algorithmic_bytes_per_launch: int):
    """HBM bytes per launch of `kernel` as the committed rocprofv3 counter summary records them
    (FETCH_SIZE + WRITE_SIZE, each scaled by what it reads for a plain copy of known size).  A run of this
    benchmark cannot read the counters itself; the record is used only if it was made for the same kernel,
    the same number of launches per step and the same algorithmic bytes per launch, otherwise the answer is
    (None, why)."""
    try:
        lines = [ln for ln in open(TRAFFIC_PROFILE) if ln.startswith("bench.py traffic record:")]
    except OSError:
        return None, "no traffic profile in profiles/"
    for ln in lines:
        f = dict(kv.split("=", 1) for kv in ln[len("bench.py traffic record:"):].split(";") if "=" in kv)
        f = {k.strip(): v.strip() for k, v in f.items()}
        if f.get("kernel") != kernel:
            continue
        if int(f["launches_per_step"]) != launches_per_step or int(f["algorithmic_bytes_per_launch"]) != algorithmic_bytes_per_launch:
            return None, "the profile's record for %s is for another launch grouping" % kernel
        return float(f["traffic_bytes_per_launch"]), "profiles/bench_resnet50_set_hbm_traffic.md (rocprofv3 FETCH_SIZE + WRITE_SIZE of this command)"
    return None, "the traffic profile has no record for %s" % kernel


WORKLOAD_NAMES = {
    0: "single 2x16x32x32 fp32 tensor, B=8 b=2 (configs[0])",
    1: "ResNet-18/CIFAR activation set, batch 128, fp32, B=4 b=2 (configs[1])",
    2: "ResNet-50/ImageNet activation set, batch 64, fp32, B=8 b=2 (configs[2])",
    3: "single 256x256x56x56 bf16 tensor, B=8 b=2 (configs[3])",
    4: "edge-shape heavy-tail fp32 set, batch 32, b=4 (configs[4])",
}


class StreamEvent:
    """A HIP event on torch's current stream, created with hipEventDisableSystemFence: recording it
    does not make the device flush its caches to system scope, which a default event (torch.cuda.Event)
    does; three bracketed launches per step cost 1.5 % of the step with default events.  The time
    stamps are the same kind.  Falls back to torch.cuda.Event when the HIP runtime cannot be reached."""
    _hip = None

    @classmethod
    def _lib(cls):
        if cls._hip is None:
            try:
                h = ctypes.CDLL("libamdhip64.so")
                h.hipEventCreateWithFlags.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint]
                h.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
                h.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
                h.hipEventDestroy.argtypes = [ctypes.c_void_p]
                cls._hip = h
            except OSError:
                cls._hip = False
        return cls._hip

    def __init__(self, torch):
        self.torch, self.ev, self.tev = torch, None, None
        h = self._lib()
        if h:
            e = ctypes.c_void_p()
            if h.hipEventCreateWithFlags(ctypes.byref(e), 0x20000000) == 0:      # hipEventDisableSystemFence
                self.ev = e
        if self.ev is None:
            self.tev = torch.cuda.Event(enable_timing=True)

    def record(self):
        if self.ev is not None:
            if self._hip.hipEventRecord(self.ev, ctypes.c_void_p(self.torch.cuda.current_stream().cuda_stream)) != 0:
                raise RuntimeError("hipEventRecord failed")
        else:
            self.tev.record()

    def elapsed_time(self, other) -> float:
        """milliseconds from this event to `other` (both recorded and complete)"""
        if self.ev is not None:
            f = ctypes.c_float()
            if self._hip.hipEventElapsedTime(ctypes.byref(f), self.ev, other.ev) != 0:
                raise RuntimeError("hipEventElapsedTime failed")
            return f.value
        return self.tev.elapsed_time(other.tev)

    def __del__(self):
        if self.ev is not None and self._hip:
            self._hip.hipEventDestroy(self.ev)


def per_shape(args, torch, pkg, dev) -> int:
    """Compress-only and decompress-only rates of every distinct shape of the workload, single calls
    and batch calls, each against a plain device copy of the map's size timed the same way."""
    from synthetic_inputs import codec_seed, draw_config

    def timed_us(fn, reps):
        """median and min over `reps` launches, each bracketed by events on the current stream"""
        for i in range(5):
            fn(i)
        ev = []
        for i in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn(i)
            e1.record()
            ev.append((e0, e1))
        torch.cuda.synchronize()
        t = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in ev)
        return t[len(t) // 2], t[0]

    groups = {}
    for k, spec, x in draw_config(args.config, args.batch):
        if spec.dtype == "bf16":
            x = x.to(torch.bfloat16)
        groups.setdefault((tuple(x.shape), x.dtype, spec.B, spec.b), []).append((k, x))
    reps = max(20, args.steps or 20)
    rows = []
    for (shape, dtype, B, b), members in groups.items():
        n = min(len(members), 8)
        nsets = max(3, args.sets)
        in_b = members[0][1].numel() * members[0][1].element_size()
        pk_b = pkg.division_packed_bytes(*shape, B, b, dtype)
        # rotating sets of n maps each, so that the last-level cache cannot hold the working set
        xs = [[torch.roll(members[j][1].to(dev), s, 0).contiguous() for j in range(n)] for s in range(nsets)]
        pk = [[torch.empty(pk_b, dtype=torch.uint8, device=dev) for _ in range(n)] for _ in range(nsets)]
        out = [[torch.empty(shape, dtype=dtype, device=dev) for _ in range(n)] for _ in range(nsets)]
        seeds = [codec_seed(args.config, members[j][0]) for j in range(n)]
        for s in range(nsets):
            pkg.division_compress_batch(xs[s], B, b, seeds, packed=pk[s])
        row = {"shape": list(shape), "dtype": "bf16" if dtype == torch.bfloat16 else "f32", "B": B, "b": b,
               "maps_in_workload": len(members), "input_bytes": in_b, "packed_bytes": pk_b,
               "compress_kernel": pkg.division_kernel_name(0, shape, B, b, dtype),
               "decompress_kernel": pkg.division_kernel_name(1, shape, B, b, dtype)}
        modes = [("single", 1)] + ([("batch", n)] if n > 1 else [])
        for name, m in modes:
            tc = timed_us(lambda i: pkg.division_compress_batch(xs[i % nsets][:m], B, b, seeds[:m], packed=pk[i % nsets][:m]), reps)
            td = timed_us(lambda i: pkg.division_decompress_batch(pk[i % nsets][:m], shape, B, b, dtype, out=out[i % nsets][:m]), reps)
            tcopy = timed_us(lambda i: [out[i % nsets][j].copy_(xs[i % nsets][j]) for j in range(m)], reps)
            alg = m * (in_b + pk_b)
            copy_gbs = 2 * m * in_b / tcopy[0] / 1e3
            row[name] = {"maps": m,
                         "compress_us_median": round(tc[0], 2), "compress_us_min": round(tc[1], 2),
                         "decompress_us_median": round(td[0], 2), "decompress_us_min": round(td[1], 2),
                         "compress_GB_s": round(alg / tc[0] / 1e3, 1), "decompress_GB_s": round(alg / td[0] / 1e3, 1),
                         "roundtrip_GB_s": round(2 * alg / (tc[0] + td[0]) / 1e3, 1),
                         "activation_GB_s": round(2 * m * in_b / (tc[0] + td[0]) / 1e3, 1),
                         "pct_hbm_peak": round(100 * 2 * alg / (tc[0] + td[0]) / 1e3 / HBM_PEAK_GBS, 1),
                         "device_copy_GB_s": round(copy_gbs, 1),
                         "roundtrip_vs_copy": round(2 * alg / (tc[0] + td[0]) / 1e3 / copy_gbs, 3)}
        row["compression_ratio"] = round(in_b / pk_b, 3)
        rows.append(row)
        del xs, pk, out
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "per-shape compress / decompress GB/s (algorithmic bytes), median of %d launches" % reps,
                      "unit": "GB/s", "n_gpus": 1, "data": "synthetic",
                      "config": {"workload": WORKLOAD_NAMES[args.config], "batch_override": args.batch},
                      "shapes": rows}))
    return 0


def masks(args, torch, pkg, dev) -> int:
    """Rates of the Relu / Dropout mask operators on maps of the workload's largest shape."""
    from synthetic_inputs import draw_config

    k, spec, x = max(draw_config(args.config, args.batch), key=lambda t: t[2].numel())
    if spec.dtype == "bf16":
        x = x.to(torch.bfloat16)
    n, es = x.numel(), x.element_size()
    nsets = max(3, args.sets)
    g = torch.Generator().manual_seed(12345)
    xs = [(torch.roll(x, s, 0) - 0.5 * (s + 1)).to(dev) for s in range(nsets)]       # mixed signs
    ys = [torch.empty_like(t) for t in xs]
    ms = [torch.empty(pkg.division_mask_bytes(n) // 4, dtype=torch.int32, device=dev) for _ in xs]
    reps = max(20, args.steps or 20)

    def timed_us(fn):
        for i in range(5):
            fn(i)
        ev = []
        for i in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn(i)
            e1.record()
            ev.append((e0, e1))
        torch.cuda.synchronize()
        t = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in ev)
        return t[len(t) // 2], t[0]

    ops = {
        "relu_forward": (lambda i: pkg.division_relu_forward(xs[i % nsets], out=ys[i % nsets], mask=ms[i % nsets]), 2 * n * es + n / 8),
        "dropout_forward": (lambda i: pkg.division_dropout_forward(xs[i % nsets], 0.5, i, out=ys[i % nsets], mask=ms[i % nsets]), 2 * n * es + n / 8),
        "mask_backward": (lambda i: pkg.division_mask_backward(ms[i % nsets], xs[i % nsets], out=ys[i % nsets]), 2 * n * es + n / 8),
        "device_copy": (lambda i: ys[i % nsets].copy_(xs[i % nsets]), 2 * n * es),
    }
    if x.dim() == 4 and x.shape[2] % 2 == 0 and x.shape[3] % 2 == 0:
        # Max-Pooling layer, k = 2: forward reads the map and writes a quarter-size map and the mask;
        # backward reads the quarter-size gradient and the mask and writes a whole map
        pooled = [pkg.division_maxpool_forward(t, 2) for t in xs]
        ops["maxpool_forward_k2"] = (lambda i: pkg.division_maxpool_forward(xs[i % nsets], 2), n * es + n * es / 4 + n / 8)
        ops["maxpool_backward_k2"] = (lambda i: pkg.division_maxpool_backward(pooled[i % nsets][1], pooled[i % nsets][0],
                                                                             tuple(x.shape), 2), n * es + n * es / 4 + n / 8)
    if x.dim() == 4 and es == 4:
        # Relu followed by the compression of its output (the conv-BN-Relu block of Theorem 3): two kernels
        # against the fused one; algorithmic bytes = x in, y out, mask, packed (+ y in again when unfused)
        sp_B, sp_b = 8, 2
        pkb = pkg.division_packed_bytes(*x.shape, sp_B, sp_b)
        pks = [torch.empty(pkb, dtype=torch.uint8, device=dev) for _ in xs]

        def two(i):
            pkg.division_relu_forward(xs[i % nsets], out=ys[i % nsets], mask=ms[i % nsets])
            pkg.division_compress(ys[i % nsets], sp_B, sp_b, i, packed=pks[i % nsets])

        ops["relu_then_compress_two_kernels"] = (two, 3 * n * es + n / 8 + pkb)
        ops["relu_compress_fused" if pkg.division_relu_compress_fused(tuple(x.shape), sp_B, sp_b) else "relu_compress_unfused_shape"] = (
            lambda i: pkg.division_relu_compress(xs[i % nsets], sp_B, sp_b, i, out=ys[i % nsets], mask=ms[i % nsets],
                                                 packed=pks[i % nsets]), 2 * n * es + n / 8 + pkb)
        # the same pair on the other shapes of the workload (one map each)
        seen = {tuple(x.shape)}
        for _, sp2, x2 in draw_config(args.config, args.batch):
            if tuple(x2.shape) in seen or x2.dim() != 4 or sp2.dtype == "bf16":
                continue
            seen.add(tuple(x2.shape))
            n2 = x2.numel()
            xs2 = [(torch.roll(x2, s, 0) - 0.5 * (s + 1)).to(dev) for s in range(nsets)]
            ys2 = [torch.empty_like(t) for t in xs2]
            ms2 = [torch.empty(pkg.division_mask_bytes(n2) // 4, dtype=torch.int32, device=dev) for _ in xs2]
            pkb2 = pkg.division_packed_bytes(*x2.shape, sp_B, sp_b)
            pks2 = [torch.empty(pkb2, dtype=torch.uint8, device=dev) for _ in xs2]
            tag = "x".join(map(str, x2.shape))
            fused2 = pkg.division_relu_compress_fused(tuple(x2.shape), sp_B, sp_b)

            def two2(i, xs2=xs2, ys2=ys2, ms2=ms2, pks2=pks2):
                pkg.division_relu_forward(xs2[i % nsets], out=ys2[i % nsets], mask=ms2[i % nsets])
                pkg.division_compress(ys2[i % nsets], sp_B, sp_b, i, packed=pks2[i % nsets])

            def one2(i, xs2=xs2, ys2=ys2, ms2=ms2, pks2=pks2):
                pkg.division_relu_compress(xs2[i % nsets], sp_B, sp_b, i, out=ys2[i % nsets], mask=ms2[i % nsets], packed=pks2[i % nsets])

            ops["relu_then_compress_two_kernels " + tag] = (two2, 3 * n2 * 4 + n2 / 8 + pkb2)
            ops[("relu_compress_fused " if fused2 else "relu_compress_unfused_shape ") + tag] = (one2, 2 * n2 * 4 + n2 / 8 + pkb2)
    res = {}
    for name, (fn, nbytes) in ops.items():
        med, mn = timed_us(fn)
        res[name] = {"us_median": round(med, 2), "us_min": round(mn, 2), "algorithmic_bytes": int(nbytes),
                     "GB_s": round(nbytes / med / 1e3, 1), "pct_hbm_peak": round(100 * nbytes / med / 1e3 / HBM_PEAK_GBS, 1)}
    for name in res:
        if name != "device_copy":
            res[name]["vs_copy"] = round(res[name]["GB_s"] / res["device_copy"]["GB_s"], 3)
    print(json.dumps({"metric": "1-bit mask operators, GB/s of algorithmic bytes (median of %d launches)" % reps,
                      "unit": "GB/s", "n_gpus": 1, "data": "synthetic", "dtype": "bf16" if es == 2 else "f32",
                      "config": {"workload": "one map %s of %s" % ("x".join(map(str, x.shape)), WORKLOAD_NAMES[args.config])},
                      "mask_bytes": pkg.division_mask_bytes(n), "cached_fraction_of_map": round(pkg.division_mask_bytes(n) / (n * es), 5),
                      "ops": res}))
    return 0


VARIANTS = [
    # what, shape, B, b     (fp32 maps; the 2-D shapes are those of the ResNet-50 set at batch 64)
    ("block size 12", (64, 256, 56, 56), 12, 2), ("block size 16", (64, 256, 56, 56), 16, 2),
    ("block size 18", (64, 256, 56, 56), 18, 2), ("block size 64", (64, 256, 56, 56), 64, 2),
    ("block size 64", (64, 512, 28, 28), 64, 2), ("block size 64", (64, 1024, 14, 14), 64, 2),
    ("block size 12", (64, 512, 28, 28), 12, 2), ("block size 18", (64, 512, 28, 28), 18, 2),
    ("block size 12", (64, 1024, 14, 14), 12, 2),
    # the sweep of Sec. 5 runs on ResNet-18 / CIFAR-10: these are its maps
    ("block size 12, CIFAR", (256, 64, 32, 32), 12, 2), ("block size 18, CIFAR", (256, 64, 32, 32), 18, 2),
    ("block size 12, CIFAR", (256, 128, 16, 16), 12, 2), ("block size 18, CIFAR", (256, 128, 16, 16), 18, 2),
    ("block size 12, CIFAR", (256, 256, 8, 8), 12, 2),
    ("8-bit codes", (64, 256, 56, 56), 8, 8), ("4-bit codes", (64, 256, 56, 56), 8, 4), ("1-bit codes", (64, 256, 56, 56), 8, 1),
    ("1-bit codes", (64, 64, 112, 112), 8, 1), ("1-bit codes", (64, 512, 28, 28), 8, 1), ("1-bit codes", (64, 1024, 14, 14), 8, 1), ("1-bit codes", (64, 2048, 7, 7), 8, 1),
    ("1-bit codes, 1-D map", (256, 128, 1, 768), 8, 1), ("1-bit codes, odd width", (256, 96, 55, 55), 8, 1),
    ("1-D map", (256, 128, 1, 768), 8, 4), ("1-D map", (64, 384, 1, 3136), 8, 4), ("1-D map", (256, 768, 1, 196), 16, 2), ("1-D map", (64, 196, 1, 3072), 64, 2),
    ("3-D map", (32, 64, 16, 56, 56), 8, 2), ("3-D map", (32, 128, 8, 28, 28), 8, 2), ("3-D map", (32, 256, 4, 14, 14), 8, 2),
    ("3-D map", (32, 512, 2, 7, 7), 8, 2), ("3-D map", (64, 64, 16, 16, 16), 8, 2), ("3-D map", (64, 64, 16, 16, 16), 4, 2),
    ("large plane", (64, 3, 224, 224), 8, 2), ("large plane", (64, 16, 224, 224), 8, 2),
    # odd widths: AlexNet's 55 x 55, 27 x 27 and 13 x 13 at batch 256, Inception-v3's 147, 73, 35 and 17 at batch 64 / 128
    ("odd width", (256, 96, 55, 55), 8, 2), ("odd width", (256, 96, 55, 55), 4, 4), ("odd width", (256, 256, 27, 27), 8, 2),
    ("odd width", (256, 384, 13, 13), 8, 2), ("odd width", (64, 64, 147, 147), 8, 2), ("odd width", (64, 96, 73, 73), 8, 2),
    ("odd width", (128, 288, 35, 35), 8, 2), ("odd width", (128, 768, 17, 17), 8, 2),
    ("odd width, block size 18", (256, 96, 55, 55), 18, 2),
]


def variants(args, torch, pkg, dev) -> int:
    """Single-call compress and decompress rates of the parameter and shape variants outside the headline
    workload: the block sizes and code widths of the paper's sweep, 1-D and 3-D maps (Appendix D), image-sized
    planes and planes of odd width."""
    nsets = max(3, args.sets)
    reps = max(20, args.steps or 20)

    def timed_us(fn):
        for i in range(3):
            fn(i)
        ev = []
        for i in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn(i)
            e1.record()
            ev.append((e0, e1))
        torch.cuda.synchronize()
        t = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in ev)
        return t[len(t) // 2]

    rows = []
    for what, shape, B, b in VARIANTS:
        g = torch.Generator(device=dev).manual_seed(sum(shape) + B)
        xs = [torch.relu(torch.randn(shape, generator=g, device=dev)) for _ in range(nsets)]
        three_d = len(shape) == 5
        nbytes = pkg.division_packed_bytes_3d(*shape, B, b) if three_d else pkg.division_packed_bytes(*shape, B, b)
        pk = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(nsets)]
        out = [torch.empty(shape, device=dev) for _ in range(nsets)]
        comp = pkg.division_compress_3d if three_d else pkg.division_compress
        dec = pkg.division_decompress_3d if three_d else pkg.division_decompress
        kn = pkg.division_kernel_name_3d if three_d else pkg.division_kernel_name
        tc = timed_us(lambda i: comp(xs[i % nsets], B, b, i, packed=pk[i % nsets]))
        td = timed_us(lambda i: dec(pk[i % nsets], shape, B, b, out=out[i % nsets]))
        tcopy = timed_us(lambda i: out[i % nsets].copy_(xs[i % nsets]))
        in_b = xs[0].numel() * 4
        alg = in_b + nbytes
        rows.append({"what": what, "shape": list(shape), "B": B, "b": b, "compression_ratio": round(in_b / nbytes, 2),
                     "compress_kernel": kn(0, shape, B, b), "decompress_kernel": kn(1, shape, B, b),
                     "compress_us": round(tc, 1), "decompress_us": round(td, 1),
                     "compress_GB_s": round(alg / tc / 1e3, 1), "decompress_GB_s": round(alg / td / 1e3, 1),
                     "device_copy_GB_s": round(2 * in_b / tcopy / 1e3, 1)})
        del xs, pk, out
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "compress / decompress GB/s (algorithmic bytes) of parameter and shape variants, single calls, median of %d" % reps,
                      "unit": "GB/s", "n_gpus": 1, "data": "synthetic", "dtype": "f32", "config": {"workload": "variants"}, "variants": rows}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default 200: 0.14 s of GPU time; the per-shape, masks and variants modes time 20 launches each)")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="workload index 0..4 (default: ResNet-50 set)")
    ap.add_argument("--sets", type=int, default=3, help="rotating buffer sets (defeats last-level-cache reuse)")
    ap.add_argument("--batch", type=int, default=None, help="override the batch size (not a valid headline run)")
    ap.add_argument("--mode", choices=["batch", "layer"], default="batch",
                    help="batch: consecutive same-shape maps share a launch (<= 8 per call); layer: one call per map")
    ap.add_argument("--c16", action="store_true",
                    help="cache H^L, delta and Delta as bfloat16 (the paper's format; fp32 workloads only)")
    ap.add_argument("--bf16", action="store_true",
                    help="every map of the workload as bfloat16 (mixed-precision training; not the headline workload)")
    ap.add_argument("--no-compare-modes", dest="compare_modes", action="store_false",
                    help="do not time the other launch mode (it is timed before the reported one and its figures go into the line)")
    ap.add_argument("--roofline-every", type=int, default=4,
                    help="bracket the dominant kernel's launches with events on every N-th timed step (default 4). "
                         "An event pair is two more packets for the command processor and opens a gap of 5-9 us "
                         "before the launch it brackets; on every step that is 4 %% of the step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-shape", action="store_true",
                    help="time compress and decompress of every distinct tensor shape of the workload on their own, "
                         "beside a plain device copy of the same size; prints one JSON line with a 'shapes' list")
    ap.add_argument("--masks", action="store_true",
                    help="time the 1-bit mask operators (Relu / Dropout forward, backward) on the largest map of the "
                         "workload, beside a plain device copy; prints one JSON line")
    ap.add_argument("--variants", action="store_true",
                    help="rates of the block sizes / code widths of the paper's sweep and of 1-D and 3-D maps")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run only a plain 1 GiB device copy 10 times (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    sub_mode = args.per_shape or args.masks or args.variants
    if args.steps is None and not sub_mode:
        args.steps = 200

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; planes are independent so data-parallel ranks would run "
              "the same kernels with no collective, but no multi-GPU figure is produced. Use --gpus 1.",
              file=sys.stderr)
        return 2

    import torch

    import paper_2208_04187_amd as pkg
    from synthetic_inputs import codec_seed, config, draw_config

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": src.numel() * 4, "copy_probe_bytes_written": src.numel() * 4,
                          "launches": 10}))
        return 0

    if args.per_shape:
        return per_shape(args, torch, pkg, dev)
    if args.masks:
        return masks(args, torch, pkg, dev)
    if args.variants:
        return variants(args, torch, pkg, dev)

    # ---- synthetic workload on the host, then resident in HBM (several rotating sets)
    _, specs = config(args.config)
    host = []
    for k, spec, x in draw_config(args.config, args.batch):
        if spec.dtype == "bf16" or args.bf16:
            x = x.to(torch.bfloat16)
        host.append((k, spec, x))
    nsets = max(1, args.sets)
    xs, packs, outs = [], [], []
    for s in range(nsets):
        xs.append([(x.to(dev) if s == 0 else torch.roll(x.to(dev), s, 0).contiguous()) for _, _, x in host])
        packs.append([torch.empty(pkg.division_packed_bytes(*x.shape, sp.B, sp.b, x.dtype, args.c16), dtype=torch.uint8, device=dev)
                      for _, sp, x in host])
        outs.append([torch.empty(x.shape, dtype=x.dtype, device=dev) for _, _, x in host])
    shapes = [tuple(x.shape) for _, _, x in host]
    dtypes = [x.dtype for _, _, x in host]
    seeds = [codec_seed(args.config, k) for k, _, _ in host]
    in_bytes = [x.numel() * x.element_size() for _, _, x in host]
    pk_bytes = [p.numel() for p in packs[0]]
    elements = sum(x.numel() for _, _, x in host)
    input_bytes, packed_bytes = sum(in_bytes), sum(pk_bytes)
    algo_bytes_step = 2 * (input_bytes + packed_bytes)

    # every launch of a step: (direction, tensor indices).  "batch": consecutive maps of one
    # shape (one stage of the network) go through the batch entry points, at most 8 per call,
    # so one call is one kernel launch; "layer": one call per map, as a layer-by-layer
    # integration issues them.
    def launch_list(mode):
        groups = []
        for i in range(len(host)):
            sp = host[i][1]
            key = (shapes[i], dtypes[i], sp.B, sp.b)
            if mode == "batch" and groups and groups[-1][0] == key and len(groups[-1][1]) < 8:
                groups[-1][1].append(i)
            else:
                groups.append((key, [i]))
        idx = [tuple(g[1]) for g in groups]
        return [(0, g) for g in idx] + [(1, g) for g in reversed(idx)]

    kname_cache = {}

    def kname(d, g):
        """kernel that serves launch (direction, maps); looked up once: the query is a host call of its own"""
        if (d, g) not in kname_cache:
            i = g[0]
            kname_cache[(d, g)] = pkg.division_kernel_name(d, shapes[i], host[i][1].B, host[i][1].b, dtypes[i], c16=args.c16)
        return kname_cache[(d, g)]

    stream = torch.cuda.current_stream().cuda_stream      # raw handle, fetched once: the per-call lookup costs the host 8 us

    def run_step(launches, s: int, timed_group=None, events=None, pool=None):
        for d, g in launches:
            sp = host[g[0]][1]
            rec = events is not None and (timed_group is None or kname(d, g) == timed_group)
            if rec:
                # events come from a pool made before the timed region: creating one costs the host
                # several microseconds, which a step of short launches would wait for
                e0 = pool.pop() if pool else StreamEvent(torch)
                e1 = pool.pop() if pool else StreamEvent(torch)
                e0.record()
            if len(g) == 1:
                i = g[0]
                if d == 0:
                    pkg.division_compress(xs[s][i], sp.B, sp.b, seeds[i], packed=packs[s][i], c16=args.c16, stream=stream)
                else:
                    pkg.division_decompress(packs[s][i], shapes[i], sp.B, sp.b, dtypes[i], out=outs[s][i], c16=args.c16, stream=stream)
            elif d == 0:
                pkg.division_compress_batch([xs[s][i] for i in g], sp.B, sp.b, [seeds[i] for i in g],
                                            packed=[packs[s][i] for i in g], c16=args.c16, stream=stream)
            else:
                pkg.division_decompress_batch([packs[s][i] for i in g], shapes[g[0]], sp.B, sp.b, dtypes[g[0]],
                                              out=[outs[s][i] for i in g], c16=args.c16, stream=stream)
            if rec:
                e1.record()
                events.append(((d, g), e0, e1))

    def timed(mode):
        launches = launch_list(mode)
        # preparation (untimed, before the warm-up): a few steps so that buffers, code objects and clocks
        # are where a running job has them, then one step that times every launch to find the dominant
        # kernel, and the events the timed region will need (creating one costs the host microseconds)
        for w in range(8):
            run_step(launches, w % nsets)
        probe = []
        run_step(launches, 0, None, probe)
        torch.cuda.synchronize()
        per_kernel = {}
        for (d, g), e0, e1 in probe:
            per_kernel[kname(d, g)] = per_kernel.get(kname(d, g), 0.0) + e0.elapsed_time(e1)
        dominant = max(per_kernel, key=per_kernel.get)
        events = []
        n_dom = sum(1 for d, g in launches if kname(d, g) == dominant)
        every = max(1, min(args.roofline_every, args.steps))
        pool = [StreamEvent(torch) for _ in range(2 * n_dom * (args.steps // every + 1))]
        # W warm-up steps, then exactly K timed steps between two synchronisations; events only around the
        # dominant kernel's launches, on every `every`-th step
        for w in range(args.warmup):
            run_step(launches, w % nsets)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            if k % every == 0:
                run_step(launches, k % nsets, dominant, events, pool)
            else:
                run_step(launches, k % nsets)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return (t1 - t0) * 1e3 / args.steps, per_kernel, dominant, events, len(launches)

    def timed_maps():
        """The whole step as two library calls (division_compress_maps, division_decompress_maps): what the
        saved-tensor hook issues when a whole forward pass fits one group.  Same protocol, no events."""
        order = list(range(len(host)))
        rev = order[::-1]
        Bs, bs = [host[i][1].B for i in order], [host[i][1].b for i in order]

        def step(s):
            pkg.division_compress_maps([xs[s][i] for i in order], Bs, bs, [seeds[i] for i in order],
                                       packed=[packs[s][i] for i in order], c16=args.c16, stream=stream)
            pkg.division_decompress_maps([packs[s][i] for i in rev], [shapes[i] for i in rev], [Bs[i] for i in rev],
                                         [bs[i] for i in rev], [dtypes[i] for i in rev], out=[outs[s][i] for i in rev],
                                         c16=args.c16, stream=stream)
        for w in range(8 + args.warmup):
            step(w % nsets)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            step(k % nsets)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    other_mode = "layer" if args.mode == "batch" else "batch"
    other_ms = timed(other_mode)[0] if args.compare_modes else None
    maps_ms = timed_maps() if args.compare_modes else None
    ms_per_step, per_kernel, dominant, events, n_launches = timed(args.mode)

    dom_ms = [e0.elapsed_time(e1) for _, e0, e1 in events]
    dom_bytes = [sum(in_bytes[i] + pk_bytes[i] for i in g) for (d, g), _, _ in events]
    avg_ms = sum(dom_ms) / len(dom_ms)
    avg_bytes = sum(dom_bytes) / len(dom_bytes)
    achieved = avg_bytes / (avg_ms * 1e-3) / 1e9
    value = algo_bytes_step / (ms_per_step * 1e-3) / 1e9

    if args.config == 2 and args.batch is None and not args.c16 and not args.bf16 and args.mode == "batch":
        n_dom_step = sum(1 for d, g in launch_list(args.mode) if kname(d, g) == dominant)
        traffic, traffic_src = recorded_traffic(dominant, n_dom_step, round(avg_bytes))
    else:
        traffic, traffic_src = None, "counters were profiled for the default workload and launch mode only"

    out = {
        "metric": "compress+decompress GB/s of activations and % of HBM peak; compression ratio",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if dtypes[0] == torch.bfloat16 else "f32",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[args.config], "tensors": len(host), "elements": elements,
                   "input_bytes": input_bytes, "packed_bytes": packed_bytes,
                   "B": host[0][1].B, "b": host[0][1].b, "buffer_sets": nsets,
                   "launch_mode": args.mode, "launches_per_step": n_launches,
                   "cache_format": "bf16 H^L, delta, Delta (Sec. 4.1)" if args.c16 else "H^L in the map's type, fp32 delta, Delta",
                   "batch_override": args.batch, "all_maps_bfloat16": bool(args.bf16)},
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "activation_GB_s": round(2 * input_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "compression_ratio": round(input_bytes / packed_bytes, 3),
        f"{other_mode}_mode_GB_s": round(algo_bytes_step / (other_ms * 1e-3) / 1e9, 1) if other_ms else None,
        f"{other_mode}_mode_ms_per_step": round(other_ms, 4) if other_ms else None,
        "maps_mode_GB_s": round(algo_bytes_step / (maps_ms * 1e-3) / 1e9, 1) if maps_ms else None,
        "maps_mode_ms_per_step": round(maps_ms, 4) if maps_ms else None,
        "kernel_ms_probe_step": {k: round(v, 4) for k, v in sorted(per_kernel.items())},
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_source": traffic_src,
                     "algorithmic_bytes_per_launch": round(avg_bytes), "avg_launch_ms": round(avg_ms, 5),
                     "launches_timed": len(dom_ms)},
    }

    # ---- CPU baseline: the oracle as it stands, on the host cores, same workload
    if not args.no_cpu_baseline and not args.c16:
        import numpy as np

        import oracle
        threads = min(16, os.cpu_count() or 1)
        tc = 0.0
        for (k, sp, x), seed in zip(host, seeds):
            if x.dtype == torch.bfloat16:
                arr, dt = x.view(torch.int16).numpy().view(np.uint16), oracle.BF16
            else:
                arr, dt = x.numpy(), oracle.F32
            a0 = time.perf_counter()
            p = oracle.compress(arr, sp.B, sp.b, seed, dt, threads=threads)
            oracle.decompress(p, tuple(x.shape), sp.B, sp.b, dt, threads=threads)
            tc += time.perf_counter() - a0
        # the same oracle on ONE thread, on the first eighth of every tensor's samples
        t1c, frac = 0.0, 0.0
        for (k, sp, x), seed in zip(host, seeds):
            ns = max(1, x.shape[0] // 8)
            xsub = x[:ns].contiguous()
            if xsub.dtype == torch.bfloat16:
                arr, dt = xsub.view(torch.int16).numpy().view(np.uint16), oracle.BF16
            else:
                arr, dt = xsub.numpy(), oracle.F32
            a0 = time.perf_counter()
            p = oracle.compress(arr, sp.B, sp.b, seed, dt, threads=1)
            oracle.decompress(p, tuple(xsub.shape), sp.B, sp.b, dt, threads=1)
            t1c += time.perf_counter() - a0
            frac += 2 * (xsub.numel() * xsub.element_size() + p.size)
        out["cpu_baseline_single_thread"] = {"value": round(frac / t1c / 1e9, 3), "unit": "GB/s", "cores": 1,
                                             "host_cores": os.cpu_count(), "kind": "oracle",
                                             "sample": f"the first eighth of the samples of every tensor, {t1c:.1f} s wall"}
        out["cpu_baseline"] = {"value": round(algo_bytes_step / tc / 1e9, 3), "unit": "GB/s", "cores": threads,
                               "host_cores": os.cpu_count(), "kind": "oracle",
                               "sample": f"one full step ({len(host)} tensors, {elements} elements) through the C oracle, "
                                         f"{threads} OpenMP threads over planes on a host that reports {os.cpu_count()} cores, {tc:.1f} s wall"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
