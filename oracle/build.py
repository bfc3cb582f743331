"""Compile the C oracle into oracle/libhdqt_oracle.so (test infrastructure only).

    python -m oracle.build
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "hdqt_oracle.c")
LIB = os.path.join(HERE, "libhdqt_oracle.so")

# -ffp-contract=off: every binary32 operation rounds on its own (no fused
# multiply-add); -fno-fast-math is gcc's default and is stated for the reader.
CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
          "-fno-fast-math", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", *CFLAGS, SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
