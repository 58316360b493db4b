"""Compile csrc/*.hip for gfx950 into paper_2210_08804_amd/libhps_cache.so (in-tree)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRCS = [os.path.join(HERE, "csrc", f) for f in ("hps_cache.hip", "hps_lookup.hip", "hps_dedup.hip", "hps_hostmap.cpp")]
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


C_DEMO_SRC = os.path.join(ROOT, "tests", "c_abi_demo.c")
C_DEMO_LIB = os.path.join(ROOT, "tests", "libhps_c_demo.so")


def build_c_demo():
    """The plain-C caller of the library that one GPU test runs (gcc, C99, no C++ anywhere)."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-pedantic", "-fPIC", "-shared",
           "-I", os.path.join(ROOT, "include"), "-isystem", os.path.join(rocm, "include"), C_DEMO_SRC, "-o", C_DEMO_LIB,
           "-L", HERE, "-l:libhps_cache.so", "-Wl,-rpath,$ORIGIN/../paper_2210_08804_amd",
           "-L", os.path.join(rocm, "lib"), "-lamdhip64"]
    subprocess.run(cmd, check=True)
    return C_DEMO_LIB


if __name__ == "__main__":
    print(build(sys.argv[1:]))
    print(build_c_demo())
