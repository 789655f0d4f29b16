"""The host side of the library (block pool, refcounted tables, split plan, in-place plan patching, blob offsets) under
AddressSanitizer and UndefinedBehaviorSanitizer, CPU only.

layout.cpp is compiled on its own with -fsanitize=address,undefined into a second shared library (no device entry
points in it), and the whole of tests/test_host_layout.py runs against that library in a child process with the
sanitizer runtime preloaded.  Any heap overflow, use after free or undefined integer / pointer operation in the index
arithmetic aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _asan_runtime():
    out = subprocess.run(["g++", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


def test_host_layout_suite_under_asan_and_ubsan():
    runtime = _asan_runtime()
    if runtime is None:
        pytest.skip("no AddressSanitizer runtime next to g++")
    sys.path.insert(0, ROOT)
    from paper_2602_12029_amd import build
    lib = build.build_host_sanitized()
    env = dict(os.environ)
    env.update({
        "PREFILLSHARE_HOST_ONLY_LIB": lib,
        "LD_PRELOAD": " ".join(filter(None, [runtime, env.get("LD_PRELOAD", "")])),
        # the interpreter's own allocations are not ours to judge; everything else stays fatal
        "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=1:halt_on_error=1",
        "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1",
    })
    # every host test except the one that asks the full library for its device symbols
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_host_layout.py"), "-k", "not exports_every_declared_symbol"],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = (res.stdout + res.stderr)[-4000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, tail
