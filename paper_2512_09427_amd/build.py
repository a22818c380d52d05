"""Builds libodma.so (host allocator + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libodma.so")
# development aids, built beside the library: a timing build whose waves stamp a clock (stream_timeline.py reads it;
# only the bf16 / head_dim 128 kernels, no prefill) and a stand-alone read probe in the attention kernel's launch shape
TIMELINE_LIB = os.path.join(HERE, "libodma_timeline.so")
DEPTH_PROBE = os.path.join(HERE, "read_depth_probe")

HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17",
    # packed fp32 forms are switched off for every kernel in this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]
# the allocator's one floating-point helper must round exactly as written
HOST_FLAGS = ["-O2", "-fPIC", "-std=c++17", "-pthread", "-ffp-contract=off", "-Wall", "-Wextra"]


def _run(cmd):
    print("+", " ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def build(verbose: bool = True) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    cxx = shutil.which("g++") or shutil.which("c++")
    if not os.path.exists(hipcc) or cxx is None:
        raise RuntimeError("hipcc and g++ are required to build libodma")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    host_o = os.path.join(obj_dir, "odma_host.o")
    dev_o = os.path.join(obj_dir, "odma_device.o")
    _run([cxx, *HOST_FLAGS, *inc, "-c", os.path.join(CSRC, "odma_host.cpp"), "-o", host_o])
    _run([hipcc, *HIP_FLAGS, *inc, "-c", os.path.join(CSRC, "odma_device.hip"), "-o", dev_o])
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", host_o, dev_o, "-pthread", "-o", LIB])
    tl_o = os.path.join(obj_dir, "odma_device_timeline.o")
    _run([hipcc, *HIP_FLAGS, "-DODMA_DEV_TIMELINE", "-DODMA_DEV_MINIMAL_VARIANTS", *inc, "-c",
          os.path.join(CSRC, "odma_device.hip"), "-o", tl_o])
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", host_o, tl_o, "-pthread", "-o", TIMELINE_LIB])
    _run([hipcc, *[f for f in HIP_FLAGS if f != "-fPIC"], os.path.join(CSRC, "read_depth_probe.hip"), "-o", DEPTH_PROBE])
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
