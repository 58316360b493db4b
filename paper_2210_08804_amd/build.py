"""Compile csrc/*.hip for gfx950 into paper_2210_08804_amd/libhps_cache.so (in-tree)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRCS = [os.path.join(HERE, "csrc", f) for f in ("hps_cache.hip", "hps_lookup.hip", "hps_dedup.hip")]
LIB = os.path.join(HERE, "libhps_cache.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # keep single-lane atomics as written: the wave-aggregating rewrite reads the result back at
    # once (readfirstlane), which puts the atomic's latency on the critical path
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    "-I", os.path.join(ROOT, "include"),
]


def build(extra=()):
    cmd = [HIPCC, *FLAGS, *extra, *SRCS, "-o", LIB, "-lpthread"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(sys.argv[1:]))
