"""The host core under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only): graph building, matching, candidate
enumeration, evaluator, row-program compiler, code generator, packs, the fusion explorer and the executors, driven over
the benchmark configurations with the launches checked by a host stub instead of run."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _asan_runtime():
    r = subprocess.run([os.environ.get("CXX", "g++"), "-print-file-name=libasan.so"], capture_output=True, text=True)
    path = r.stdout.strip()
    if r.returncode == 0 and os.path.isabs(path) and os.path.exists(path):
        return os.path.realpath(path)
    found = sorted(glob.glob("/usr/lib/x86_64-linux-gnu/libasan.so.*"))
    return found[0] if found else None


def test_host_core_is_clean_under_asan_and_ubsan():
    runtime = _asan_runtime()
    if runtime is None:
        pytest.skip("the host compiler's AddressSanitizer runtime is not installed")
    from paper_2009_10924_amd.build import build_host_sanitized
    lib = build_host_sanitized()
    env = dict(os.environ, FUSION_STITCHING_LIB=lib, LD_PRELOAD=runtime, FS_CODEGEN_CACHE_DIR="",
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1:halt_on_error=1", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    env.pop("FS_STUB_COMPILE_OK", None)
    r = subprocess.run([sys.executable, os.path.join(ROOT, "tests", "host_sanitizer_driver.py")], env=env, capture_output=True, text=True,
                       timeout=900)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "no report" in r.stdout and "ERROR: AddressSanitizer" not in r.stderr and "runtime error:" not in r.stderr, tail
