"""Compile the C part of the oracle with gcc (test infrastructure; see package docstring)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "cs_oracle.c")
LIB = os.path.join(HERE, "libcs_oracle.so")


def build(force: bool = False) -> str:
    """Build ``libcs_oracle.so`` next to its source; returns the library path."""
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", SRC, "-o", tmp, "-lm"])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
