"""Compile the CPU oracle (plain C, gcc) into oracle/libspotlight_oracle.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "spotlight_oracle.c")
# SPOTLIGHT_ORACLE_LIB: load (and build into) another file, e.g. a sanitizer build of the same source
LIB = os.environ.get("SPOTLIGHT_ORACLE_LIB") or os.path.join(HERE, "libspotlight_oracle.so")

# -ffp-contract=off: only the fused multiply-adds written as fmaf() are fused.
FLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
         "-fno-fast-math", "-mfma", "-msse4.1", "-Wall", "-Wextra"]


def build(force: bool = True, out: str = None, extra_flags=()) -> str:
    out = out or LIB
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
        return out
    subprocess.run(["gcc", *FLAGS, *extra_flags, "-o", out, SRC, "-lm"], check=True)
    return out


if __name__ == "__main__":
    print(build())
