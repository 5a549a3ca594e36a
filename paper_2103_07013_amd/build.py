"""Builds libbps.so (the C-ABI batch renderer) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbps.so")
SOURCES = ["bps_api.hip", "raster_kernels.hip", "shade_kernels.hip", "clusters.cpp"]
HEADERS = ["raster_kernels.h", "raster_device.h", "clusters.h", os.path.join("..", "..", "include", "bps.h")]
# -ffp-contract=off: the numeric rule fixes where fused multiply-adds happen.
# packed FP32 instructions are switched off on purpose (hipcc's host pass does not know the
# feature and says so; that message is harmless).
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source into paper_2103_07013_amd/libbps.so."""
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *[os.path.join(CSRC, f) for f in SOURCES], "-o", LIB]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libbps.so:\n" + res.stdout)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
