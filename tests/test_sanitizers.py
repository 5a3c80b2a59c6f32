"""CPU-side hygiene: the oracle's pins and the library's host-only argument checks run once more
against AddressSanitizer + UndefinedBehaviorSanitizer builds (host code only; no GPU is involved)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]


def _runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True, check=True).stdout.strip()
    if not os.path.isabs(path):
        pytest.skip(f"{name} not installed")
    return path


def _env(runtimes, **extra):
    env = dict(os.environ)
    preload = [p for p in env.get("LD_PRELOAD", "").split(":") if p]      # whatever is preloaded stays
    env["LD_PRELOAD"] = ":".join(preload + list(runtimes))
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(extra)
    return env


def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    from oracle import build as oracle_build
    lib = oracle_build.build(out=str(tmp_path / "libspotlight_oracle_san.so"), extra_flags=SAN)
    files = sorted(os.path.join(ROOT, "tests", f) for f in os.listdir(os.path.join(ROOT, "tests"))
                   if f.startswith("test_oracle_") and f.endswith(".py"))
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files],
                         env=_env([_runtime("libasan.so"), _runtime("libubsan.so")], SPOTLIGHT_ORACLE_LIB=lib), cwd=ROOT, capture_output=True, text=True)
    tail = (run.stdout + run.stderr)[-3000:]
    assert run.returncode == 0, tail
    assert "runtime error" not in tail and "AddressSanitizer" not in tail, tail


def test_host_side_of_the_abi_passes_under_sanitizers(tmp_path):
    """The library's host code (configuration checks, workspace planning, argument checks of every
    entry point) compiled with the sanitizers, without kernels; tests/test_abi.py runs against it."""
    from paper_2508_19740_amd import build as hip_build
    lib = str(tmp_path / "libspotlight_san.so")
    rt = hip_build.build_host_sanitized(lib)
    if not rt:
        pytest.skip("clang's AddressSanitizer runtime is not installed")
    assert hip_build.built_id(lib) == hip_build.source_id()
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_abi.py")],
                         env=_env([rt], SPOTLIGHT_LIB=lib), cwd=ROOT, capture_output=True, text=True)
    tail = (run.stdout + run.stderr)[-3000:]
    assert run.returncode == 0, tail
    assert "runtime error" not in tail and "AddressSanitizer" not in tail and "building" not in tail, tail
