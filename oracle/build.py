"""Compile the C++ twin of the CPU oracle (oracle/cq_oracle.cpp) into oracle/libcq_oracle.so.

Plain g++ with OpenMP; no flag that lets the compiler reassociate or contract floating point
(-O2 only, -ffp-contract=off), so every sum runs in the order the source states."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "cq_oracle.cpp")
LIB_PATH = os.path.join(HERE, "libcq_oracle.so")


def build_oracle(force: bool = True) -> str:
    if not force and os.path.exists(LIB_PATH) and os.path.getmtime(LIB_PATH) >= os.path.getmtime(SRC):
        return LIB_PATH
    cxx = shutil.which("g++") or shutil.which("c++")
    if cxx is None:
        raise RuntimeError("no C++ compiler found; the oracle twin cannot be built")
    cmd = [cxx, "-O2", "-std=c++17", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
           "-shared", "-Wall", "-o", LIB_PATH, SRC]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("building the oracle twin failed:\n%s\n%s" % (r.stdout, r.stderr))
    if r.stderr.strip():
        sys.stderr.write(r.stderr)
    return LIB_PATH


if __name__ == "__main__":
    print(build_oracle())
