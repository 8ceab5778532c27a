"""Build libgosh.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgosh.so")
EXAMPLE_SRC = os.path.join(HERE, "examples", "embed_example.cpp")
EXAMPLE = os.path.join(HERE, "examples", "embed_example")

SOURCES = ["gosh_host.cpp", "gosh_coarsen.cpp", "gosh_sampler.cpp", "gosh_coarsen_gpu.hip", "gosh_train.hip", "gosh_embed.hip", "gosh_parts.hip", "gosh_place.hip"]

FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    "-fopenmp",
    "-Wall",
    "-Wno-unused-function",
    # fp32 atomic adds on coarse-grained device memory use the hardware instruction
    "-munsafe-fp-atomics",
    # packed-fp32 instructions are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: libgosh needs the ROCm toolchain")
    return exe


def build(verbose: bool = False) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    cmd = [hipcc(), *FLAGS, "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
           "-x", "hip", *srcs, "-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    build_example(verbose)
    return LIB


def build_example(verbose: bool = False) -> str:
    """The C++ program that uses the library through include/gosh.h alone."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wall",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I" + os.path.join(ROOT, "include"), EXAMPLE_SRC, "-L" + HERE, "-lgosh",
           "-Wl,-rpath,$ORIGIN/..", "-o", EXAMPLE]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return EXAMPLE


if __name__ == "__main__":
    print(build(verbose=True))
