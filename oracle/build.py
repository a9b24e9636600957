"""Compile the CPU oracle (oracle/obref.cpp) into oracle/libobref.so with g++.

Test infrastructure only.  Contraction is off so that every binary32 operation rounds once.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "obref.cpp")
LIB = os.path.join(HERE, "libobref.so")
FLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
         "-pthread", "-Wall", "-Wextra"]


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
            os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "obref.h"))):
        return LIB
    cmd = ["g++"] + FLAGS + [SRC, "-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
