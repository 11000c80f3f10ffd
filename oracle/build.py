"""Compile the CPU oracle (test infrastructure) into oracle/liboracle_cser.so with g++.

Contraction is switched off so that every fused multiply-add in the oracle is one that
its source spells out.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(HERE, "cser_oracle.cpp")
LIBRARY = os.path.join(HERE, "liboracle_cser.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIBRARY) and os.path.getmtime(LIBRARY) >= os.path.getmtime(SOURCE):
        return LIBRARY
    cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
           "-shared", "-fPIC", SOURCE, "-o", LIBRARY + ".tmp"]
    subprocess.run(cmd, check=True)
    os.replace(LIBRARY + ".tmp", LIBRARY)
    return LIBRARY


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
