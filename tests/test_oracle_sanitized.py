"""The oracle and its pins under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

The oracle is built a second time with -fsanitize=address,undefined and the pin tests, the
generator's margin tests and an argument-error sweep run against that build in a child process
(the sanitizer runtime has to be the first library of a process, so it cannot be loaded into
this one).  Any out-of-bounds access, use of freed memory, signed overflow or misaligned access
in the oracle's C code aborts the child.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    out = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True)
    path = out.stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("no AddressSanitizer runtime beside gcc")
    sys.path.insert(0, ROOT)
    from oracle import build as oracle_build
    library = oracle_build.build_sanitized(str(tmp_path / "libppow_oracle_san.so"))
    env = dict(os.environ)
    preload = [asan] + [p for p in env.get("LD_PRELOAD", "").split(":") if p]
    env.update(LD_PRELOAD=":".join(preload), PPOW_ORACLE_LIBRARY=library,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1",     # Python itself leaks by design
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", OMP_NUM_THREADS="4")
    run = subprocess.run(
        [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
         os.path.join(ROOT, "tests", "test_oracle_pins.py"),
         os.path.join(ROOT, "tests", "test_workloads.py")],
        cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (run.stdout + run.stderr)[-3000:]
    assert run.returncode == 0, tail
    assert "passed" in run.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
