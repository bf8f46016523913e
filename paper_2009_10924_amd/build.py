"""Builds libfusion_stitching.so for gfx950 with hipcc, in-tree.

`python -m paper_2009_10924_amd.build` or `build()`; cross-compiles without a GPU.
"""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
OBJ_DIR = os.path.join(CSRC, "build")
LIB_PATH = os.path.join(PKG_DIR, "libfusion_stitching.so")

SOURCES = [
    "fs_graph.cpp", "fs_unfused.cpp", "fs_match.cpp", "fs_cost.cpp", "fs_stitch.cpp", "fs_family_softmax.cpp", "fs_family_layernorm.cpp", "fs_family_gelu.cpp",
    "fs_family_transpose.cpp", "fs_family_rows.cpp", "fs_plan.cpp", "fs_pack.cpp", "fs_rowprog.cpp", "fs_explore.cpp", "fs_program.cpp", "fs_codegen.cpp",
    "kernels/launch.hip", "kernels/unfused.hip", "kernels/softmax.hip", "kernels/layernorm.hip",
    "kernels/gelu.hip", "kernels/tchain.hip", "kernels/rowops.hip", "kernels/pack.hip", "kernels/rowprog.hip",
    "kernels/gen_runtime.hip", "kernels/gen_sample.hip", "kernels/static_scratch.hip", "kernels/stream_probe.hip",
]

# device headers the run-time compiler gets as text in front of a generated kernel: (file, name of the C string)
EMBEDDED = [("kernels/device_utils.hpp", "kEmbeddedDeviceUtils"), ("kernels/gen_support.hpp", "kEmbeddedGenSupport")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function"]
# packed-fp32 VALU ops stay off (some of their forms misbehave on the test machines)
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-command-line-argument"]


def _compile(src: str, verbose: bool) -> str:
    obj = os.path.join(OBJ_DIR, src.replace("/", "_") + ".o")
    path = os.path.join(CSRC, src)
    if src.endswith(".hip"):
        cmd = [HIPCC, *COMMON, *DEVICE, "-c", path, "-o", obj]
    else:
        cmd = [HIPCC, *COMMON, "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-c", path, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l and l.strip() != "1 warning generated when compiling for host.")
    if r.returncode != 0:
        raise RuntimeError(f"compile failed: {src}\n{err}")
    if err.strip() and verbose:
        print(err, file=sys.stderr)
    return obj


def _embed_sources() -> None:
    """csrc/build/embedded_sources.inc: each embedded header as a raw string literal, without `#pragma once`
    and without its includes of the library's own headers (their text is concatenated in order instead)."""
    parts = []
    for rel, name in EMBEDDED:
        with open(os.path.join(CSRC, rel)) as f:
            lines = [l for l in f.read().splitlines() if l.strip() != "#pragma once" and not l.startswith('#include "')]
        text = "\n".join(lines) + "\n"
        assert ')FSRC"' not in text
        parts.append(f'static const char {name}[] = R"FSRC({text})FSRC";\n')
    path = os.path.join(OBJ_DIR, "embedded_sources.inc")
    new = "".join(parts)
    old = open(path).read() if os.path.exists(path) else None
    if new != old:
        with open(path, "w") as f:
            f.write(new)


def build(verbose: bool = False, jobs: int | None = None) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    _embed_sources()
    jobs = jobs or min(8, len(SOURCES), os.cpu_count() or 1)
    with cf.ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(lambda s: _compile(s, verbose), SOURCES))
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB_PATH, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed\n{r.stderr}")
    return LIB_PATH


HOST_SAN_LIB = os.path.join(PKG_DIR, "libfusion_stitching_host_san.so")


def build_host_sanitized(verbose: bool = False) -> str:
    """TEST-ONLY: the host core (every .cpp of SOURCES) with csrc/host_stub.cpp in place of the HIP kernels, built by
    the host compiler with AddressSanitizer and UndefinedBehaviorSanitizer.  Needs no GPU and no ROCm; a process that
    loads it preloads the compiler's libasan (tests/test_host_sanitizers.py does).  Launches are checked and counted,
    never run."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    _embed_sources()
    cxx = os.environ.get("CXX", "g++")
    flags = ["-O1", "-g", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-fsanitize=address,undefined",
             "-fno-omit-frame-pointer", "-fno-sanitize-recover=undefined"]
    srcs = [s for s in SOURCES if s.endswith(".cpp")] + ["host_stub.cpp"]

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ_DIR, "san_" + src.replace("/", "_") + ".o")
        cmd = [cxx, *flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"sanitizer build of the host core failed: {src}\n{r.stderr}")
        return obj

    with cf.ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        objs = list(pool.map(compile_one, srcs))
    r = subprocess.run([cxx, "-shared", "-fsanitize=address,undefined", "-o", HOST_SAN_LIB, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"sanitizer link of the host core failed\n{r.stderr}")
    return HOST_SAN_LIB


if __name__ == "__main__":
    if "--host-sanitized" in sys.argv:
        print(build_host_sanitized(verbose="-v" in sys.argv))
    else:
        print(build(verbose="-v" in sys.argv))
