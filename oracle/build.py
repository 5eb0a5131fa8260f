"""Compile the plain-C oracle (oracle/la_oracle.c) into oracle/libla_oracle.so with gcc.

Test infrastructure only.  Building the checker is not using it: the build entry
point compiles it, and the ctypes wrapper rebuilds it when the source is newer.
"""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "la_oracle.c")
LIB = os.path.join(_HERE, "libla_oracle.so")


def build(force: bool = False) -> str:
    stale = (not os.path.exists(LIB)) or os.path.getmtime(LIB) < os.path.getmtime(SRC)
    if force or stale:
        tmp = LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", tmp, SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
