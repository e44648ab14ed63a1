"""Builds libdivision.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
from pathlib import Path

PKG = Path(__file__).resolve().parent
SRCS = [PKG / "csrc" / "division.hip", PKG / "csrc" / "masks.hip"]
LIB = PKG / "libdivision.so"

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17",
    "-ffp-contract=off",                       # fp32 steps of the codec are never fused
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fPIC", "-shared",
    "-Rpass-analysis=kernel-resource-usage",   # parsed below: no kernel may spill to scratch
]


def build(verbose: bool = False) -> Path:
    """Compile unconditionally; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB.with_name(LIB.name + ".tmp%d" % os.getpid())
    cmd = [hipcc, *HIPCC_FLAGS, "-o", str(tmp), *map(str, SRCS)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    spills = [ln for ln in res.stderr.splitlines()
              if "ScratchSize [bytes/lane]:" in ln and not ln.split("ScratchSize [bytes/lane]:")[1].strip().startswith("0")]
    if spills:
        tmp.unlink(missing_ok=True)
        raise RuntimeError("a kernel spills registers to scratch memory (performance guard):\n" + "\n".join(spills[:5]))
    if verbose and res.stderr:
        print("\n".join(ln for ln in res.stderr.splitlines() if "remark:" not in ln))
    os.replace(tmp, LIB)
    return LIB
