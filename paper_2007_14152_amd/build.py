"""Compile the HIP library for gfx950 in-tree (csrc/libspdnn.so)."""
from __future__ import annotations

import os
import re
import subprocess
import sys

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


NO_SCRATCH_KERNELS = ["fused_row2_kernel", "fused_pair_kernel"]


def _resource_usage(text):
    """Per kernel (mangled name): the figures of the compiler's -Rpass-analysis=kernel-resource-usage remarks."""
    out, cur = {}, None
    for line in text.splitlines():
        m = re.search(r"remark: +Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark: +([A-Za-z \[\]/]+): (\d+)", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return out


def build(verbose: bool = False, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-Rpass-analysis=kernel-resource-usage"] + list(extra) + SOURCES + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    usage = _resource_usage(res.stderr)
    if res.returncode != 0:
        sys.stderr.write("\n".join(l for l in res.stderr.splitlines() if "kernel-resource-usage" not in l) + "\n")
        raise subprocess.CalledProcessError(res.returncode, cmd)
    # Kernels that issue their global loads as inline instructions keep the loaded values in registers
    # the compiler believes to be ready; a spill between load and wait would save stale data.
    for kernel in NO_SCRATCH_KERNELS:
        hits = {k: v for k, v in usage.items() if kernel in k}
        if not hits:
            raise RuntimeError("build check: kernel %s not found in the compiler's resource report" % kernel)
        for k, v in hits.items():
            if v.get("ScratchSize [bytes/lane]", 0) != 0:
                raise RuntimeError("build check: %s uses %d bytes of scratch per lane; it must use none"
                                   % (k, v["ScratchSize [bytes/lane]"]))
    if verbose:
        for k, v in sorted(usage.items()):
            if "fused_" in k:
                print("%s: VGPRs %s, scratch %s B/lane" % (k, v.get("VGPRs"), v.get("ScratchSize [bytes/lane]")))
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
