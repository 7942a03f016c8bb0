"""Compile the C oracle into ``oracle/libnpd_oracle.so`` with gcc (host only)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "npd_oracle.c")
LIB = os.path.join(HERE, "libnpd_oracle.so")


def compile_source(src: str, lib: str) -> str:
    # -O2 without -ffast-math: sums stay in the order they are written.
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra", "-o", lib, src, "-lm"]
    subprocess.check_call(cmd)
    return lib


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    return compile_source(SRC, LIB)


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
