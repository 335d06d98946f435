"""Compile the HIP library for gfx950 into paper_1806_03461_amd/libtfhe_mi355x.so.

hipcc cross-compiles without a GPU.  The library is built in-tree so that it travels with
the source tree; nothing is installed.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtfhe_mi355x.so")
SOURCES = ["host_keys.cpp", "executor.cpp", "bnn_lower.cpp", "kernels.hip"]


def build(verbose: bool = False) -> str:
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
           "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose="-v" in sys.argv))
