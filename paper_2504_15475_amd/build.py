"""Compile the HIP library in-tree for gfx950: paper_2504_15475_amd/libersd.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "ersd_race.hip")
SRC_HOST = os.path.join(HERE, "csrc", "ersd_tree.cpp")  # host-only part of the library
SRC_GSD = os.path.join(HERE, "csrc", "ersd_gsd.hip")    # the comparison method
SRC_GSD_TREE = os.path.join(HERE, "csrc", "ersd_gsd_tree.hip")  # the comparison method on a draft tree
LIB = os.path.join(HERE, "libersd.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 instructions are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off",  # fp64 scores are evaluated exactly as written; fmaf() calls stay explicit
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"),
]


def build(extra=()):
    rounds = os.environ.get("ERSD_PHILOX_ROUNDS")  # 7 by default (set in the source); 10 = the generator's standard
    if rounds:
        extra = (*extra, f"-DERSD_PHILOX_ROUNDS={int(rounds)}")
    cmd = [HIPCC, *FLAGS, *extra, "-o", LIB, SRC, SRC_GSD, SRC_GSD_TREE, SRC_HOST]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
