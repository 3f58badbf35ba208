"""Compile the CPU oracle (test infrastructure) into oracle/libqkvref.so with g++."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, "qkv_ref.cpp"), os.path.join(HERE, "controller_ref.cpp"),
        os.path.join(HERE, "inject_ref.cpp")]
LIB = os.path.join(HERE, "libqkvref.so")


def build(force=True):
    """Build the shared library; returns its path.  With force=False an up-to-date one is kept."""
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(s) for s in SRCS):
        return LIB
    cmd = ["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", "-o", LIB] + SRCS
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
