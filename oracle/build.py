"""Compile the C++ oracle into oracle/libdaf_oracle.so with the host compiler.

The flags matter for parity: no contraction into fused multiply-add, no fast-math, so
every written operation rounds once in IEEE binary32.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "daf_oracle.cpp")
LIB = os.path.join(HERE, "libdaf_oracle.so")
FLAGS = ["-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
         "-shared", "-fPIC"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["g++", *FLAGS, "-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
    sys.exit(0)
