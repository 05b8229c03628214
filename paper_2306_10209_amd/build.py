"""Compile the HIP kernels + C ABI into paper_2306_10209_amd/lib/libzpp_gfx950.so.

gfx950 only.  -ffp-contract=off keeps every fp32 operation separately rounded
(the bit-exactness contract of include/zpp.h); packed-fp32 instruction selection
is switched off for the device pass.
"""
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
SRC = os.path.join(PKG, "csrc", "zpp_gfx950.hip")
INC = os.path.join(ROOT, "include")
LIBDIR = os.path.join(PKG, "lib")
LIB = os.path.join(LIBDIR, "libzpp_gfx950.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fPIC", "-shared", "-Wall", "-Wno-unused-command-line-argument", f"-I{INC}"]


def build(force: bool = True, extra=()) -> str:
    os.makedirs(LIBDIR, exist_ok=True)
    deps = [SRC, os.path.join(INC, "zpp.h"), os.path.join(INC, "zpp_diagnostics.h")]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    cmd = [HIPCC, *FLAGS, *extra, SRC, "-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True, extra=sys.argv[1:]))
