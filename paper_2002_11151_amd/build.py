"""Builds the HIP library (csrc/*.hip -> libxbar.so beside this file) for gfx950 with hipcc: one object
per source file, compiled side by side, then one link."""
import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = [os.path.join(HERE, "csrc", name) for name in ("vmm_f16_a.hip", "vmm_f16_b.hip", "vmm_f6_a.hip", "vmm_f6_b.hip", "xbar.hip", "wire.hip",
                                                     "fcm.hip", "pulse.hip", "periph.hip")]
LIB = os.path.join(HERE, "libxbar.so")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include")]


def build(verbose=False):
    extra = ["-Rpass-analysis=kernel-resource-usage"] if verbose else []
    with tempfile.TemporaryDirectory() as tmp:
        objects = [os.path.join(tmp, os.path.basename(s) + ".o") for s in SRC]

        def compile_one(pair):
            subprocess.run(["hipcc"] + FLAGS + extra + ["-c", "-o", pair[1], pair[0]], check=True)

        with ThreadPoolExecutor(max_workers=min(len(SRC), os.cpu_count() or 1)) as pool:
            list(pool.map(compile_one, zip(SRC, objects)))
        subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objects, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
