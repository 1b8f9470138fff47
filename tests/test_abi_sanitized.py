"""The host side of the C ABI under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

libppow is built a second time with the sanitizers on its host code (device code as usual) and
the ABI tests -- exported symbols, struct layouts, workspace queries and every argument error
that returns before a launch -- run against that build in a child process (the sanitizer runtime
has to be the first library of a process).  Any out-of-bounds access, overflow or misaligned
access in the argument checks or the workspace arithmetic aborts the child.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_abi_tests_pass_with_a_host_sanitized_library(tmp_path):
    sys.path.insert(0, ROOT)
    from paper_2605_14978_amd import build as ppow_build
    runtime = ppow_build.sanitizer_runtime()
    if runtime is None:
        pytest.skip("no shared AddressSanitizer runtime beside hipcc's compiler")
    library = ppow_build.build_host_sanitized(str(tmp_path / "libppow_san.so"))
    env = dict(os.environ)
    preload = [runtime] + [p for p in env.get("LD_PRELOAD", "").split(":") if p]
    env.update(LD_PRELOAD=":".join(preload), PPOW_LIBRARY=library,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1",     # Python itself leaks by design
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    run = subprocess.run(
        [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
         os.path.join(ROOT, "tests", "test_abi.py")],
        cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    tail = (run.stdout + run.stderr)[-3000:]
    assert run.returncode == 0, tail
    assert "passed" in run.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
