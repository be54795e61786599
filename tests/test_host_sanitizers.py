"""The library's host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no kernel runs).

The host side holds the index arithmetic that no parity test sees: Algorithm 1 / Algorithm 2 and the tracker's
bookkeeping in rserve_sched.cpp (section 3.1 - 3.3), and in rserve_prefill.hip the descriptor sizing, the staging ring,
the page lists and the argument checks that a host-only context runs before any launch.  The test builds the library a
second time with both sanitizers on the host pass (paper_2509_24381_amd.build.build(sanitize_host_to=...)) and runs
tests/test_scheduler.py and tests/test_abi_host.py against that build in a child process that has the ASan runtime
preloaded; any report (heap overflow, use after free, signed overflow, misaligned access, ...) aborts the child.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r"""
import sys
import paper_2509_24381_amd.binding as b
b.library_path = lambda: sys.argv[1]          # the instrumented build instead of the in-tree library
import pytest
sys.exit(pytest.main(["-x", "-q", "-p", "no:cacheprovider", "tests/test_scheduler.py", "tests/test_abi_host.py"]))
"""


@pytest.mark.sanitizer
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    from paper_2509_24381_amd import build
    lib = build.build(verbose=False, sanitize_host_to=str(tmp_path / "librserve_prefill_asan.so"))
    symbols = subprocess.run(["nm", "-D", lib], capture_output=True, text=True, check=True).stdout
    assert "__asan_report" in symbols and "__ubsan_handle" in symbols, "the build is not instrumented"
    env = dict(os.environ)
    # the runtime must be first among the preloaded libraries; whatever is preloaded already stays behind it
    env["LD_PRELOAD"] = build.asan_runtime() + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # (leak checking off: the interpreter itself never frees much of what it allocates)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    proc = subprocess.run([sys.executable, "-c", CHILD, lib], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (proc.stdout + proc.stderr)[-4000:]
    assert proc.returncode == 0, tail
    assert "passed" in proc.stdout and "failed" not in proc.stdout, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
