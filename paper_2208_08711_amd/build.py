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


def build_c_example(verbose: bool = False) -> str:
    """tests/native/abi_roundtrip.c -> abi_roundtrip.bin: the ABI used from plain C (gcc, C99),
    linked against libl3.so and the HIP runtime.  A GPU test runs it."""
    src = os.path.join(ROOT, "tests", "native", "abi_roundtrip.c")
    out = os.path.join(ROOT, "tests", "native", "abi_roundtrip.bin")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-Wall", "-O1", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"), src, "-o", out,
           "-L", HERE, "-l:libl3.so", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_2208_08711_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_c_example(verbose=True))
    sys.exit(0)
