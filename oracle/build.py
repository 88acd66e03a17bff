"""Compile the CPU oracle (test infrastructure) into oracle/libq8_oracle.so.

Q8_ORACLE_SRC names another C source to compile instead (the mutation tests build altered
copies of the oracle this way, next to that source); nothing else reads it."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.environ.get("Q8_ORACLE_SRC") or os.path.join(HERE, "q8_oracle.c")
LIB = (os.path.splitext(SRC)[0] + ".so") if os.environ.get("Q8_ORACLE_SRC") else os.path.join(HERE, "libq8_oracle.so")
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, SRC, "-lm"])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
