"""Builds libdivision.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

division.hip (with the kernel families and the host side in the .h fragments it includes) instantiates
its kernels once per element / cache type; it is compiled as three translation units (-DDIVISION_PART=0, 1, 2: float, bfloat16, bfloat16-cached float) beside masks.hip,
all four in parallel, and the objects are linked into the one library.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
DIVISION = PKG / "csrc" / "division.hip"
MASKS = PKG / "csrc" / "masks.hip"
SRCS = [DIVISION, MASKS]
LIB = PKG / "libdivision.so"
# (object name, source, extra flags)
UNITS = [
    ("division_f32.o", DIVISION, ["-DDIVISION_PART=0"]),
    ("division_bf16.o", DIVISION, ["-DDIVISION_PART=1"]),
    ("division_c16.o", DIVISION, ["-DDIVISION_PART=2"]),
    ("masks.o", MASKS, []),
]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17",
    "-ffp-contract=off",                       # fp32 steps of the codec are never fused
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fPIC",
    "-Rpass-analysis=kernel-resource-usage",   # parsed below: no kernel may spill to scratch
]


def build(verbose: bool = False, extra_flags=(), out: Path | None = None) -> Path:
    """Compile unconditionally; returns the path of the shared library.  extra_flags are added to every
    hipcc compile line and out replaces the library's path (both for builds that compare variants)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    lib_path = Path(out) if out is not None else LIB
    objdir = Path(tempfile.mkdtemp(prefix="division_build_"))
    try:
        def compile_unit(unit):
            name, src, extra = unit
            cmd = [hipcc, *HIPCC_FLAGS, *extra, *extra_flags, "-c", "-o", str(objdir / name), str(src)]
            return name, subprocess.run(cmd, capture_output=True, text=True)

        with ThreadPoolExecutor(max_workers=len(UNITS)) as pool:
            results = list(pool.map(compile_unit, UNITS))
        for name, res in results:
            if res.returncode != 0:
                raise RuntimeError("hipcc failed on %s:\n%s" % (name, res.stderr))
        log = "".join(res.stderr for _, res in results)
        spills = [ln for ln in log.splitlines()
                  if "ScratchSize [bytes/lane]:" in ln and not ln.split("ScratchSize [bytes/lane]:")[1].strip().startswith("0")]
        if spills:
            raise RuntimeError("a kernel spills registers to scratch memory (performance guard):\n" + "\n".join(spills[:5]))
        if verbose and log:
            print("\n".join(ln for ln in log.splitlines() if "remark:" not in ln))
        tmp = lib_path.with_name(lib_path.name + ".tmp%d" % os.getpid())
        link = [hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", str(tmp), *(str(objdir / u[0]) for u in UNITS)]
        res = subprocess.run(link, capture_output=True, text=True)
        if res.returncode != 0:
            tmp.unlink(missing_ok=True)
            raise RuntimeError("link failed:\n" + res.stderr)
        os.replace(tmp, lib_path)
    finally:
        shutil.rmtree(objdir, ignore_errors=True)
    return lib_path
