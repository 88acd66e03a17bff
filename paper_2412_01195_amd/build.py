"""Build the C-ABI library (hipcc, gfx950) into paper_2412_01195_amd/libq8opt.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libq8opt.so")
SOURCES = [os.path.join(CSRC, "q8opt_kernels.hip"), os.path.join(CSRC, "q8opt_host.cpp")]
HEADERS = [os.path.join(CSRC, "q8opt_internal.h"), os.path.join(ROOT, "include", "q8opt.h")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # no fused multiply-add in the update formulas
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fvisibility=hidden", "-Wall",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(force: bool = True, extra=()) -> str:
    if force or stale():
        tmp = LIB + ".tmp.%d" % os.getpid()
        cmd = [HIPCC, *FLAGS, *extra, "-o", tmp]
        for s in SOURCES:
            cmd += ["-x", "hip", s]
        subprocess.check_call(cmd)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
