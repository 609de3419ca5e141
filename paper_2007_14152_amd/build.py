"""Compile the HIP library for gfx950 in-tree (csrc/libspdnn.so)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(CSRC, "libspdnn.so")
SOURCES = [os.path.join(CSRC, "spdnn.hip")]
HEADERS = [os.path.join(CSRC, "spdnn_kernels.h"), os.path.join(CSRC, "spdnn_order.h"),
           os.path.join(CSRC, "spdnn_layout.h"),
           os.path.join(os.path.dirname(_HERE), "include", "spdnn.h")]
# host build of the connection-ordering routine, for tests of the set-up logic without a GPU
ORDER_HOST_LIB = os.path.join(CSRC, "libspdnn_order_host.so")
ORDER_HOST_SRC = os.path.join(CSRC, "spdnn_order_host.cpp")

# Packed-FP32 instructions are switched off for all device code.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + list(extra) + SOURCES + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    subprocess.run(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-o", ORDER_HOST_LIB, ORDER_HOST_SRC],
                   check=True)
    return LIB


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build(verbose=True))
