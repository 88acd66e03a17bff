"""Build the C-ABI library (hipcc, gfx950) into paper_2412_01195_amd/libq8opt.so.

Five objects are compiled in parallel -- the host translation unit (entry points, quantize /
dequantize kernels), the optimizer-step kernels once per storage type of w and g (float,
bfloat16, binary16; same source, different -D), and the host-only table builder -- and linked
into one shared library.  A sixth object, the benchmark's traffic probe, is linked together
with the same five into a second library, libq8opt_probe.so, which only bench.py loads (for
its workload probe1b); the product library does not contain it.
"""
import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libq8opt.so")
PROBE_LIB = os.path.join(HERE, "libq8opt_probe.so")
HEADERS = [os.path.join(CSRC, "q8opt_internal.h"), os.path.join(CSRC, "q8opt_device.h"), os.path.join(CSRC, "q8opt_exact.h"),
           os.path.join(ROOT, "include", "q8opt.h")]
# (object name, source, extra defines)
UNITS = [
    ("kernels", os.path.join(CSRC, "q8opt_kernels.hip"), []),
    ("steps_f32", os.path.join(CSRC, "q8opt_steps.hip"), ["-DQ8_STEPS_F32"]),
    ("steps_bf16", os.path.join(CSRC, "q8opt_steps.hip"), ["-DQ8_STEPS_BF16"]),
    ("steps_f16", os.path.join(CSRC, "q8opt_steps.hip"), ["-DQ8_STEPS_F16"]),
    ("host", os.path.join(CSRC, "q8opt_host.cpp"), []),
]
PROBE_UNIT = ("probe", os.path.join(CSRC, "q8opt_probe.hip"), [])
SOURCES = sorted({u[1] for u in UNITS + [PROBE_UNIT]})
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
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


def build(force: bool = True, extra=(), out: str = LIB, jobs: int = 6) -> str:
    if not (force or stale()):
        return out
    probe_out = os.path.join(os.path.dirname(out), "libq8opt_probe.so")
    tmpdir = tempfile.mkdtemp(prefix="q8opt_build_")
    try:
        def compile_unit(unit):
            name, src, defs = unit
            obj = os.path.join(tmpdir, name + ".o")
            subprocess.check_call([HIPCC, *FLAGS, *extra, *defs, "-c", "-x", "hip", src, "-o", obj])
            return obj
        with ThreadPoolExecutor(max(1, jobs)) as pool:
            objs = list(pool.map(compile_unit, UNITS + [PROBE_UNIT]))
        for target, members in ((out, objs[:-1]), (probe_out, objs)):
            tmp = target + ".tmp.%d" % os.getpid()
            subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *members])
            os.replace(tmp, target)
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)
    return out


if __name__ == "__main__":
    print(build(force=True))
