"""Builds libshe_hip.so (HIP kernels + C ABI) for gfx950 next to this file."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libshe_hip.so")
SOURCES = ["she_kernels.hip", "she_api.cpp", "she_host.cpp", "she_circuits.cpp", "she_leveled.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-pthread",
    # keep hipcc from forming packed FP32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-result", "-Wno-unused-value",
]


def build(verbose: bool = False, extra: list[str] | None = None, out: str | None = None) -> str:
    """Compiles every source each time it is called; returns the path of the shared library."""
    out = out or LIB_PATH
    cmd = [HIPCC] + FLAGS + (extra or []) + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", out + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd, stderr=None if verbose else subprocess.DEVNULL)
    os.replace(out + ".tmp", out)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
