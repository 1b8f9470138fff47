"""Compile the oracle (plain C, double precision) into oracle/libppow_oracle.so.

Test infrastructure: the product path never loads this library.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(HERE, "ppow_oracle.c")
LIBRARY = os.path.join(HERE, "libppow_oracle.so")


SANITIZED_LIBRARY = os.path.join(HERE, "libppow_oracle_san.so")


def build_sanitized(output: str = SANITIZED_LIBRARY) -> str:
    """Build the oracle with AddressSanitizer and UndefinedBehaviorSanitizer (host code only).

    A process that loads the result needs the ASan runtime first in its library list:
    LD_PRELOAD=$(gcc -print-file-name=libasan.so), and PPOW_ORACLE_LIBRARY=<this file> to make
    the oracle package use it.
    """
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-o", output, SOURCE, "-lm"]
    subprocess.run(cmd, check=True, cwd=HERE)
    return output


def build(force: bool = True) -> str:
    """Build the shared library and return its path.

    With force=False an up-to-date library is kept.  PPOW_ORACLE_LIBRARY names a library
    built elsewhere (the sanitizer build) to be used as it is.
    """
    if os.environ.get("PPOW_ORACLE_LIBRARY"):
        return os.environ["PPOW_ORACLE_LIBRARY"]
    header = os.path.join(HERE, "ppow_oracle.h")
    if not force and os.path.exists(LIBRARY):
        newest = max(os.path.getmtime(SOURCE), os.path.getmtime(header))
        if os.path.getmtime(LIBRARY) >= newest:
            return LIBRARY
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           "-o", LIBRARY, SOURCE, "-lm"]
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIBRARY


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
