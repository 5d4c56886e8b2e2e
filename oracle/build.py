"""Compile the CPU oracle (plain C, gcc) into oracle/libfc_oracle.so.

Test infrastructure only: nothing in the GPU product path imports this.
"""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "fc_oracle.c")
LIB = os.path.join(_HERE, "libfc_oracle.so")
CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Build the shared library; returns its path."""
    stale = (not os.path.exists(LIB)) or os.path.getmtime(LIB) < os.path.getmtime(SRC)
    if force or stale:
        tmp = LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", *CFLAGS, SRC, "-o", tmp, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
