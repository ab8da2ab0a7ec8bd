"""The host side of the C ABI (argument validation, launch planning, workspace sizing: everything
that runs before a kernel is enqueued) under AddressSanitizer + UndefinedBehaviorSanitizer: the
library is built once more with the sanitizers on its host code and the host-only ABI tests run
against that build in a child process that preloads the sanitizer runtime.  No GPU is touched."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_abi_host_paths_under_asan_and_ubsan():
    rt = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not rt:
        pytest.skip("the compiler's AddressSanitizer runtime is not installed")
    from paper_2508_16201_amd import build
    lib = build.LIB_HOSTSAN
    newest = max(os.path.getmtime(f) for f in build.sources() + glob.glob(os.path.join(build.HERE, "csrc", "*.h")) +
                 [os.path.join(ROOT, "include", "specvlm.h")])
    if not os.path.exists(lib) or os.path.getmtime(lib) < newest:
        build.build(host_sanitizers=True)
    env = dict(os.environ)
    env.update({
        "SPECVLM_LIB": lib,
        # the sanitizer runtime must come first in the list; whatever was preloaded stays behind it
        "LD_PRELOAD": ":".join(x for x in (rt[0], os.environ.get("LD_PRELOAD", "")) if x),
        "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=1:halt_on_error=1:protect_shadow_gap=0",
        "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1",
    })
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_abi.py"],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
