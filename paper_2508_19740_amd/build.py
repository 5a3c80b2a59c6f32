"""Compile the HIP library for gfx950 into paper_2508_19740_amd/libspotlight.so (in-tree)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.environ.get("SPOTLIGHT_LIB") or os.path.join(HERE, "libspotlight.so")
SOURCES = ["api.hip", "hash.hip", "retrieve.hip", "attend.hip"]

# -ffp-contract=off: the hash codes are defined by an exact sequence of binary32 operations, so
#   only the fused multiply-adds written out in the source may be fused.
# -packed-fp32-ops off: the compiler must not form packed binary32 instructions.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-fno-fast-math", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes"]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, "internal.h"), os.path.join(ROOT, "include", "spotlight.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = False) -> str:
    """One hipcc per source file, side by side, then the link."""
    import concurrent.futures
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    compile_flags = [f for f in FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory(prefix="spotlight_build_") as tmp:
        objs = [os.path.join(tmp, os.path.basename(src) + ".o") for src in sources()]

        def compile_one(pair):
            src, obj = pair
            cmd = [hipcc, *compile_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd))
            subprocess.run(cmd, check=True)

        with concurrent.futures.ThreadPoolExecutor(max_workers=len(objs)) as pool:
            list(pool.map(compile_one, zip(sources(), objs)))
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
