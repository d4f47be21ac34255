"""Builds the HIP library (csrc/*.hip -> libxbar.so beside this file) for gfx950 with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = [os.path.join(HERE, "csrc", "xbar.hip"), os.path.join(HERE, "csrc", "periph.hip")]
LIB = os.path.join(HERE, "libxbar.so")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include")]


def build(verbose=False):
    cmd = ["hipcc"] + FLAGS + (["-Rpass-analysis=kernel-resource-usage"] if verbose else []) + ["-o", LIB] + SRC
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
