"""Build liblbt.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblbt.so")
PEAKS = os.path.join(HERE, "lbt_peaks")        # stand-alone probe of the chip's ceilings
SOURCES = ["lbt_api.hip", "lbt_quantize.hip", "lbt_gemm.hip", "lbt_profile.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                       # codes are decided by un-fused fp32 arithmetic
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    if not os.path.exists(PEAKS) or os.path.getmtime(PEAKS) < os.path.getmtime(os.path.join(CSRC, "lbt_peaks.hip")):
        return True
    deps = sources() + [os.path.join(CSRC, "lbt_internal.h"), os.path.join(ROOT, "include", "lbt.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", tmp] + sources()
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    build_peaks(hipcc, verbose)
    return LIB


def build_peaks(hipcc=None, verbose: bool = False) -> str:
    """The peak probe `bench.py --peaks` runs (an executable beside the library)."""
    hipcc = hipcc or os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = PEAKS + ".tmp.%d" % os.getpid()
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", tmp, os.path.join(CSRC, "lbt_peaks.hip")]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    os.replace(tmp, PEAKS)
    return PEAKS


if __name__ == "__main__":
    print(build(force=True, verbose=True))
