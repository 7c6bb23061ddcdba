"""Build libsradamw.so (HIP, gfx950) in-tree with hipcc.

Flags that decide bit-exactness: -ffp-contract=off (no FMA contraction of the
update's separate multiplies and adds); correctly rounded FP32 divide and sqrt
and FP32 subnormal support are hipcc's defaults and are left on.  Packed FP32
instructions are disabled for device code.
"""
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsradamw.so")
SOURCES = [os.path.join(CSRC, "sradamw.hip")]
HEADERS = [os.path.join(CSRC, "sr_kernels.h"), os.path.join(CSRC, "sr_device.h"), os.path.join(CSRC, "sr_host.h"),
           os.path.join(os.path.dirname(HERE), "include", "sradamw.h")]

HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
         "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def is_fresh() -> bool:
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    return all(os.path.getmtime(f) <= t for f in SOURCES + HEADERS)


def build(force: bool = True, extra=()) -> str:
    if not force and is_fresh():
        return LIB
    cmd = [HIPCC, *FLAGS, *extra, *SOURCES, "-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True, extra=sys.argv[1:]))
