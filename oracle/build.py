"""Build the oracle shared library (test infrastructure, not the product).

    python oracle/build.py

Compiles oracle/l3_oracle.cpp with the host C++ compiler into
oracle/libl3_oracle.so.  No GPU, no ROCm.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "l3_oracle.cpp")
OUT = os.path.join(HERE, "libl3_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= max(
            os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "l3_oracle.h"))):
        return OUT
    cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", OUT, SRC]
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
