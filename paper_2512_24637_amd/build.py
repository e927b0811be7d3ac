"""Builds libmsched.so (HIP, gfx950) in-tree with hipcc."""
import glob
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libmsched.so")
SOURCES = sorted(glob.glob(os.path.join(PKG, "csrc", "*.hip")))
HEADERS = sorted(glob.glob(os.path.join(PKG, "csrc", "*.h"))) + [os.path.join(ROOT, "include", "msched.h")]


TIMERS_LIB = os.path.join(PKG, "libmsched_timers.so")


def build(force: bool = True, timers: bool = False) -> str:
    """Compile every HIP source for gfx950 into one shared library.  timers=True builds a second library,
    libmsched_timers.so, whose planning kernels record the wall clock at their phase boundaries (a tuning aid:
    nothing loads it unless told to)."""
    lib = TIMERS_LIB if timers else LIB
    if not force and os.path.exists(lib):
        newest = max(os.path.getmtime(p) for p in SOURCES + HEADERS)
        if os.path.getmtime(lib) >= newest:
            return lib
    # -packed-fp32-ops: the device pass takes the feature (no packed fp32 instructions are formed); only the host
    # pass, which knows no such feature, prints "not a recognized feature for this target" - harmless.
    cmd = ["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-o", lib] + (["-DMSCHED_KERNEL_TIMERS"] if timers else []) + SOURCES
    subprocess.check_call(cmd)
    return lib


if __name__ == "__main__":
    print(build())
