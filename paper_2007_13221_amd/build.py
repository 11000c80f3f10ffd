"""Compile the HIP library for gfx950 into paper_2007_13221_amd/libcser_hip.so (in-tree).

hipcc cross-compiles without a GPU.  Flags: contraction off (every fused multiply-add in the
kernels is written out, so results do not depend on the optimiser's choices) and packed-fp32
instruction selection off.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
SOURCES = [os.path.join(CSRC, "cser_kernels.hip"), os.path.join(CSRC, "cser_api.hip")]
HEADERS = [os.path.join(CSRC, "cser_internal.h"), os.path.join(os.path.dirname(HERE), "include", "cser.h"),
           os.path.join(os.path.dirname(HERE), "include", "cser_measure.h")]
LIBRARY = os.path.join(HERE, "libcser_hip.so")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument"]


def up_to_date() -> bool:
    if not os.path.exists(LIBRARY):
        return False
    built = os.path.getmtime(LIBRARY)
    return all(os.path.getmtime(f) <= built for f in SOURCES + HEADERS)


def build(force: bool = True, extra_flags=()) -> str:
    if not force and up_to_date():
        return LIBRARY
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + list(extra_flags) + SOURCES + ["-o", LIBRARY + ".tmp"]
    subprocess.run(cmd, check=True)
    os.replace(LIBRARY + ".tmp", LIBRARY)
    return LIBRARY


if __name__ == "__main__":
    print(build(force=True, extra_flags=sys.argv[1:]))
