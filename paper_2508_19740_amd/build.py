"""Compile the HIP library for gfx950 into paper_2508_19740_amd/libspotlight.so (in-tree).

The library carries the hash of the sources it was built from (spotlight_build_id); stale()
compares it with the sources in the tree, so a library older than its sources is rebuilt, not run.
"""
import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.environ.get("SPOTLIGHT_LIB") or os.path.join(HERE, "libspotlight.so")
OBJDIR = os.path.join(HERE, "_build")          # object files of the last build (not tracked)
HEADERS = [os.path.join(CSRC, h) for h in sorted(os.listdir(CSRC)) if h.endswith(".h")] + [
           os.path.join(ROOT, "include", "spotlight.h")]
ID_MARK = "SPOTLIGHT_BUILD_ID="

# -ffp-contract=off: the hash codes are defined by an exact sequence of binary32 operations, so
#   only the fused multiply-adds written out in the source may be fused.
# -packed-fp32-ops off: the compiler must not form packed binary32 instructions.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-fno-fast-math", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes"]


def sources():
    return sorted(os.path.join(CSRC, s) for s in os.listdir(CSRC) if s.endswith(".hip"))


def _digest(paths, extra=""):
    h = hashlib.sha256(extra.encode())
    for p in paths:
        h.update(os.path.basename(p).encode())
        with open(p, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def source_id() -> str:
    """Hash of every source, header and compiler flag the library is built from."""
    return _digest(sources() + [h for h in HEADERS if os.path.exists(h)], " ".join(FLAGS))


def built_id(path: str = None):
    """The source hash recorded inside a built library (read from the file, not by loading it)."""
    path = path or LIB
    if not os.path.exists(path):
        return None
    with open(path, "rb") as f:
        blob = f.read()
    at = blob.find(ID_MARK.encode())
    if at < 0:
        return None
    return blob[at + len(ID_MARK):at + len(ID_MARK) + 16].decode(errors="replace")


def stale() -> bool:
    return built_id() != source_id()


def build(verbose: bool = False, force: bool = True) -> str:
    """One hipcc per source file, side by side, then the link.  With force=False the object files
    of sources that have not changed since the last build are reused."""
    import concurrent.futures
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJDIR, exist_ok=True)
    sid = source_id()
    headers = [h for h in HEADERS if os.path.exists(h)]
    jobs = []
    objs = []
    for src in sources():
        key = _digest([src] + headers, " ".join(FLAGS) + sid * (os.path.basename(src) == "api.hip"))
        obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
        objs.append(obj)
        tag = obj + ".key"
        have = open(tag).read() if os.path.exists(tag) and os.path.exists(obj) else None
        if force or have != key:
            jobs.append((src, obj, tag, key))

    def compile_one(job):
        src, obj, tag, key = job
        if os.path.exists(tag):
            os.remove(tag)
        cmd = [hipcc, *FLAGS, f'-DSPOTLIGHT_BUILD_ID_STRING="{ID_MARK}{sid}"', "-I", os.path.join(ROOT, "include"),
               "-I", CSRC, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        with open(tag, "w") as f:
            f.write(key)

    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as pool:
        list(pool.map(compile_one, jobs))
    # stale objects of sources that no longer exist must not be linked
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB + ".tmp", *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


def build_host_sanitized(out: str) -> str:
    """The library with its HOST code (argument checks, planning, launch logic) compiled with
    AddressSanitizer and UndefinedBehaviorSanitizer, the kernels left alone: for running the
    host-only ABI tests under them.  Returns the sanitizer runtime that has to be preloaded into
    the process that loads the library."""
    import concurrent.futures
    import glob
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all"]
    with tempfile.TemporaryDirectory(prefix="spotlight_san_") as tmp:
        def one(src):
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            subprocess.run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-ffp-contract=off",
                            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *san, f'-DSPOTLIGHT_BUILD_ID_STRING="{ID_MARK}{source_id()}"',
                            "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj], check=True)
            return obj
        with concurrent.futures.ThreadPoolExecutor(max_workers=8) as pool:
            objs = list(pool.map(one, sources()))
        subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined", "-fno-gpu-sanitize",
                        "-shared-libsan", "-o", out, *objs], check=True)
    rt = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    return rt[0] if rt else ""


if __name__ == "__main__":
    import sys
    print(build(verbose=True, force="--incremental" not in sys.argv))
    print("build id", built_id())
