"""Compile the C oracle into oracle/libtorq_oracle.so with gcc.

Test infrastructure only: the product never loads this library.
Run as `python -m oracle.build` or call `build()`.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libtorq_oracle.so")


def build(force: bool = True) -> str:
    src = os.path.join(HERE, "torq_oracle.c")
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
            os.path.getmtime(src), os.path.getmtime(os.path.join(HERE, "torq_oracle.h"))):
        return LIB
    # -ffp-contract=off: no fused multiply-adds, so every product and sum is
    # rounded as the C source says.
    cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-Wall", "-Wextra", "-o", LIB, src, "-lm"]
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build())
