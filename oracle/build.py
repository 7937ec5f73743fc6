"""Compile the C oracle into oracle/liboracle.so with gcc (test infrastructure only)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, "preserve_oracle.c"), os.path.join(HERE, "preserve_oracle_q8.c")]
HDR = os.path.join(HERE, "preserve_oracle.h")
LIB = os.path.join(HERE, "liboracle.so")


def build(force: bool = False) -> str:
    stale = (not os.path.exists(LIB)
             or os.path.getmtime(LIB) < max(os.path.getmtime(f) for f in SRCS + [HDR]))
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-ffp-contract=off", "-o", LIB] + SRCS + ["-lm"]
        subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
