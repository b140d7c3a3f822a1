"""Build the CPU oracle's shared library (test infrastructure; never part of the product path)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "sc_oracle.cpp")
LIB = os.path.join(HERE, "libsc_oracle.so")


def build(force: bool = False, src: str = SRC, lib: str = LIB) -> str:
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(src):
        return lib
    cmd = ["g++", "-std=c++17", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", lib, src]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(force=True))
