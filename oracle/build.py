"""Compile the CPU oracle (plain C, gcc) into oracle/libsfo.so.  Test infrastructure only."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libsfo.so")


def build(force: bool = False) -> str:
    src = os.path.join(HERE, "sfo.c")
    hdr = os.path.join(HERE, "sfo.h")
    if not force and os.path.exists(LIB):
        if os.path.getmtime(LIB) >= max(os.path.getmtime(src), os.path.getmtime(hdr)):
            return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", LIB, src, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
