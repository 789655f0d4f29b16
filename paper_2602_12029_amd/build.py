"""Compile the HIP/C++ sources into paper_2602_12029_amd/libprefillshare.so for gfx950.

Every source becomes an object file of its own (compiled in parallel, under `_build/`), then one link.
`python -m paper_2602_12029_amd.build --sanitize` builds the host side alone (block pool, tables, split
plan: layout.cpp) with AddressSanitizer and UBSan into libprefillshare_host_asan.so for the CPU-only
sanitizer test; the device entry points are absent from that library.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = ["layout.cpp", "abi.hip", "wave_attention.hip", "mfma_attention.hip", "prefill_attention.hip", "merge.hip",
           "kv_update.hip", "probe.hip"]
LIB = os.path.join(HERE, "libprefillshare.so")
HOST_ASAN_LIB = os.path.join(HERE, "libprefillshare_host_asan.so")
OBJ_DIR = os.path.join(HERE, "_build")
INCLUDES = ["-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc")]


def _run(cmd, verbose=False):
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(" ".join(cmd) + "\n" + res.stdout + res.stderr)
        raise RuntimeError("compiler failed: " + os.path.basename(cmd[-3] if len(cmd) > 3 else cmd[0]))
    if verbose:
        sys.stderr.write(res.stderr)


def build(verbose: bool = False, jobs: int = 0) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"] + INCLUDES
    objects = [os.path.join(OBJ_DIR, os.path.splitext(s)[0] + ".o") for s in SOURCES]

    def compile_one(pair):
        src, obj = pair
        _run([hipcc] + flags + ["-c", os.path.join(HERE, "csrc", src), "-o", obj], verbose)

    jobs = jobs or min(len(SOURCES), max(1, min(16, len(os.sched_getaffinity(0)))))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(compile_one, zip(SOURCES, objects)))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objects + ["-o", LIB], verbose)
    return LIB


def build_host_sanitized(verbose: bool = False) -> str:
    """The host side (no HIP call in it) under AddressSanitizer + UndefinedBehaviorSanitizer, for CPU-only tests."""
    cxx = os.environ.get("CXX", "g++")
    _run([cxx, "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-fno-omit-frame-pointer",
          "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"] + INCLUDES +
         [os.path.join(HERE, "csrc", "layout.cpp"), "-o", HOST_ASAN_LIB], verbose)
    return HOST_ASAN_LIB


if __name__ == "__main__":
    if "--sanitize" in sys.argv:
        print(build_host_sanitized(verbose="-v" in sys.argv))
    else:
        print(build(verbose="-v" in sys.argv))
