"""Compile the C part of the CPU oracle (test infrastructure) with gcc.

`python -m oracle.build` or `oracle.build.build()`; the shared object lands
next to the source and is loaded by oracle/accept.py through ctypes.
"""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "accept.c")
LIB = os.path.join(_HERE, "liboracle_accept.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
           "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
