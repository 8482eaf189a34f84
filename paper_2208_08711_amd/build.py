"""Build the HIP library for gfx950 in-tree: paper_2208_08711_amd/libl3.so.

    python -m paper_2208_08711_amd.build

hipcc cross-compiles without a GPU.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libl3.so")
SOURCES = [os.path.join(CSRC, "l3_host.cpp"), os.path.join(CSRC, "l3_device.hip"),
           os.path.join(CSRC, "l3_encode.hip"), os.path.join(CSRC, "l3_ablation.hip")]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-ffp-contract=off",
           # packed FP32 instructions are kept out of every HIP object of this library
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-x", "hip", *SOURCES, "-o", OUT]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
