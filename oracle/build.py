"""Compile the CPU oracle (plain C, OpenMP) into oracle/librib_oracle.so.

Test infrastructure only.  Run as `python oracle/build.py`; the loader in
oracle/__init__.py also calls build() when the library is missing or older than
its source.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "rib_oracle.c")
LIB = os.path.join(HERE, "librib_oracle.so")


def build(force: bool = False) -> str:
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
