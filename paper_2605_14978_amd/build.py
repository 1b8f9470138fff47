"""Compile the HIP sources of libppow for gfx950 into paper_2605_14978_amd/libppow.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIBRARY = os.path.join(HERE, "libppow.so")
SOURCES = ["api.hip", "row_stats.hip", "row_cluster.hip", "window_epilogue.hip", "select.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
    # logits are finite by contract: lets max/min compile without NaN quieting moves
    "-fno-honor-nans",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build(verbose: bool = False, defines=(), output: str = LIBRARY) -> str:
    """Compile every HIP source and link the shared library; returns its path.

    `defines` (e.g. ["PPOW_ROW_UNROLL=8"]) and `output` build a tuning variant elsewhere.
    """
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd += ["-D" + d for d in defines]
    cmd += [os.path.join(CSRC, s) for s in SOURCES] + ["-o", output]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True, cwd=HERE)
    return output


def sanitizer_runtime():
    """Path of clang's shared AddressSanitizer runtime beside hipcc's compiler, or None."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = subprocess.run([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"],
                         capture_output=True, text=True)
    path = out.stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def build_host_sanitized(output: str) -> str:
    """The same library with AddressSanitizer + UndefinedBehaviorSanitizer on its HOST code only
    (argument checks, workspace arithmetic, launch set-up); device code is built as usual.  For
    CPU-side tests: load it in a process that has sanitizer_runtime() preloaded."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f != "-O3"] + ["-O1", "-g", "-shared-libsan"]
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"):
        flags += ["-Xarch_host", f]
    cmd = [hipcc] + flags + ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd += [os.path.join(CSRC, s) for s in SOURCES] + ["-o", output]
    subprocess.run(cmd, check=True, cwd=HERE)
    return output


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
