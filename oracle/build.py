"""Compile the CPU oracle (test infrastructure) into oracle/libqsdp_ref.so with gcc.

Strict binary32 semantics: no contraction, no fast-math. Run as
``python oracle/build.py`` or call :func:`build`.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "qsdp_ref.c")
LIB = os.path.join(HERE, "libqsdp_ref.so")

CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
          "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
            os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "qsdp_ref.h"))):
        return LIB
    cmd = ["gcc"] + CFLAGS + [SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build())
