"""Compile the CPU oracle (test infrastructure) into oracle/liboracle.so with g++.

Flags: -O2, no fast-math, -ffp-contract=off (the Pong comparison is bit for bit, so no fused
multiply-add may be formed).  Run as `python oracle/build_oracle.py`.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ["philox.cpp", "pong.cpp", "body.cpp", "cartpole.cpp"]
LIB = os.path.join(HERE, "liboracle.so")


def build(force=True, src_dir=None, out=None):
    """src_dir / out: build another copy of the sources into another library (the mutation test
    compiles deliberately broken copies this way); the defaults are the in-tree ones."""
    src_dir = src_dir or HERE
    lib = out or LIB
    srcs = [os.path.join(src_dir, s) for s in SOURCES if os.path.exists(os.path.join(src_dir, s))]
    if not force and os.path.exists(lib) and all(
            os.path.getmtime(lib) >= os.path.getmtime(s) for s in srcs):
        return lib
    cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
           "-pthread", "-Wall", "-Wextra", "-o", lib] + srcs + ["-lm"]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
