"""Compile the CPU oracle (plain C, gcc) into oracle/libsfo.so.  Test infrastructure only."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libsfo.so")


def build(force: bool = False, sanitize: bool = False, out: str = None) -> str:
    """-> path of the shared library.  SFO_LIB in the environment names a library built elsewhere (the
    sanitizer run of the tests); sanitize=True builds with AddressSanitizer + UBSan into `out`."""
    if os.environ.get("SFO_LIB") and not sanitize:
        return os.environ["SFO_LIB"]
    src = os.path.join(HERE, "sfo.c")
    if sanitize:
        cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-fsanitize=address,undefined",
               "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", out, src, "-lm"]
        subprocess.run(cmd, check=True)
        return out
    hdr = os.path.join(HERE, "sfo.h")
    if not force and os.path.exists(LIB):
        if os.path.getmtime(LIB) >= max(os.path.getmtime(src), os.path.getmtime(hdr)):
            return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", LIB, src, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
