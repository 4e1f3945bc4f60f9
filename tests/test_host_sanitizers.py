"""The host side of the library (pool bookkeeping, attention and relocation plans, handle selection,
eviction bookkeeping, the MIAD controller, the wake-up gate) under AddressSanitizer and
UndefinedBehaviorSanitizer: the host tests that need no GPU are run once more, in a child process,
against a build of the same sources whose host code is instrumented."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST_TESTS = ["tests/test_abi.py", "tests/test_policy.py", "tests/test_golden.py"]


def test_host_tests_pass_under_address_and_undefined_sanitizers():
    from paper_2604_07874_amd import build as B
    try:
        runtime = B.asan_runtime()
    except RuntimeError as e:
        pytest.skip(str(e))
    lib = B.HOSTSAN_LIB
    newest = max(os.path.getmtime(p) for p in B.source_paths())
    if not os.path.exists(lib) or os.path.getmtime(lib) < newest:
        B.build_host_sanitized(verbose=False)
    env = dict(os.environ)
    env["VALVEKV_LIBRARY"] = lib
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1"       # the interpreter itself is not leak-clean
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    res = subprocess.run([sys.executable, "-m", "pytest", *HOST_TESTS, "-m", "not gpu", "-x", "-q", "-p", "no:cacheprovider"],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    text = res.stdout + res.stderr
    assert res.returncode == 0, text[-4000:]
    assert "AddressSanitizer" not in text and "runtime error:" not in text, text[-4000:]
    assert " passed" in text
