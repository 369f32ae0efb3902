"""Compile the C oracle into oracle/libersd_oracle.so with gcc (host only, OpenMP over rows)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ersd_oracle.c")
LIB = os.path.join(HERE, "libersd_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
        os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "ersd_oracle.h"))
    ):
        return LIB
    # -ffp-contract=off: no fused multiply-adds, so the fp64 arithmetic is exactly as written
    rounds = os.environ.get("ERSD_PHILOX_ROUNDS")  # same switch as the GPU library's build
    defs = [f"-DORACLE_PHILOX_ROUNDS={int(rounds)}"] if rounds else []
    cmd = ["gcc", *defs, "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build())
