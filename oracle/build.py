"""Compile the oracle (plain C, double precision) into oracle/libppow_oracle.so.

Test infrastructure: the product path never loads this library.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(HERE, "ppow_oracle.c")
LIBRARY = os.path.join(HERE, "libppow_oracle.so")


def build(force: bool = True) -> str:
    """Build the shared library and return its path.

    With force=False an up-to-date library is kept.
    """
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
