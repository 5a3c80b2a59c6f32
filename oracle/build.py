"""Compile the CPU oracle (plain C, gcc) into oracle/libspotlight_oracle.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "spotlight_oracle.c")
LIB = os.path.join(HERE, "libspotlight_oracle.so")

# -ffp-contract=off: only the fused multiply-adds written as fmaf() are fused.
FLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
         "-fno-fast-math", "-mfma", "-msse4.1", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    subprocess.run(["gcc", *FLAGS, "-o", LIB, SRC, "-lm"], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
