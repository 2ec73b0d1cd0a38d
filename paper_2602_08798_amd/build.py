"""Compile the HIP library for gfx950 into paper_2602_08798_amd/libcryptogen_hip.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "cryptogen.hip")
LIB = os.path.join(HERE, "libcryptogen_hip.so")
DEPS = [SRC] + [os.path.join(HERE, "csrc", f) for f in ("kernels.hpp", "tables.hpp", "modarith.hpp")] + [
    os.path.join(os.path.dirname(HERE), "include", "cryptogen_bench.h"),
    os.path.join(os.path.dirname(HERE), "include", "cryptogen.h")]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # products and sums must round separately (explicit fma only)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(force: bool = True, extra=()) -> str:
    if not force and os.path.exists(LIB) and all(
            os.path.getmtime(LIB) >= os.path.getmtime(d) for d in DEPS):
        return LIB
    cmd = ["hipcc"] + FLAGS + list(extra) + ["-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True, extra=sys.argv[1:]))
