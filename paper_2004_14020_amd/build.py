"""Compile the HIP library for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libcaramel.so")
SOURCES = ["plan.cpp", "schedule.cpp", "tiles.cpp", "kernels.hip", "probe.hip", "api.hip"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


# Packed fp32 arithmetic is switched off for the device code.  The switch is an AMDGPU target
# feature, so only the gfx950 pass of hipcc takes it (checked by tests/test_build_flags.py: the
# device assembly holds no packed fp32 instruction); the host (x86-64) pass does not know the
# feature and says so once per source, which build() drops from the compiler's output.
DEVICE_FEATURE = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
HOST_PASS_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"


def flags() -> list:
    return ["-std=c++17", "-O3", "--offload-arch=gfx950", "-ffp-contract=off", "-fno-fast-math", *DEVICE_FEATURE,
            "-Wall", "-Wno-unused-command-line-argument",
            "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]


def command() -> list:
    src = [os.path.join(HERE, "csrc", s) for s in SOURCES]
    return [hipcc(), *flags(), "-fPIC", "-shared", *src, "-o", LIB]


def build(verbose: bool = True) -> str:
    cmd = command()
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = res.stdout.splitlines()
    kept = [l for l in lines if HOST_PASS_NOTE not in l]
    if kept:
        print("\n".join(kept), flush=True)
    if verbose and len(kept) != len(lines):
        print(f"({len(lines) - len(kept)} notes of the host pass about the device-only feature switch dropped)", flush=True)
    if res.returncode:
        raise subprocess.CalledProcessError(res.returncode, cmd)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
