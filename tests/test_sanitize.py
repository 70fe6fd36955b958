"""Host code of the library under AddressSanitizer and UndefinedBehaviorSanitizer, CPU only.

The argument-validation tests of tests/test_abi.py (NULL pointers, bad shapes, workspace sizes, variant
feasibility, launch-plan queries: everything an entry point does before it launches) are run once more in a
child interpreter that loads the sanitized build of the library (build.py --sanitize) with the sanitizer
runtime preloaded.  No GPU is touched: those tests return before any launch."""
import os
import subprocess
import sys

import pytest

from paper_2407_20496_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _sanitized_library() -> str:
    lib = build.SANITIZE_LIB
    newest = max(os.path.getmtime(os.path.join(d, f)) for d in (build.CSRC, os.path.join(ROOT, "include"))
                 for f in os.listdir(d))
    if not os.path.exists(lib) or os.path.getmtime(lib) < newest:
        build.build(verbose=False, sanitize=True)
    return lib


@pytest.mark.timeout(900)
def test_abi_validation_under_asan_and_ubsan():
    lib = _sanitized_library()
    runtime = build.sanitizer_runtime()
    assert os.path.exists(runtime), runtime
    syms = subprocess.run(["nm", "-D", lib], capture_output=True, text=True, check=True).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms, "the library was not built with the sanitizers"
    env = dict(os.environ)
    env["LD_PRELOAD"] = ":".join(x for x in (runtime, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1"      # the interpreter itself is not leak-clean
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["HINM_LIBRARY"] = lib
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_abi.py"), "-q", "-x",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    out = res.stdout + res.stderr
    assert res.returncode == 0, out[-4000:]
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert " passed" in out
