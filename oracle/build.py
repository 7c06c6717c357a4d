"""Compile the C part of the CPU oracle (test infrastructure, not product code)."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtsm_oracle.so")
SRC_PATH = os.path.join(_HERE, "conv_direct.c")


def build(force=False):
    """gcc -O2 -fopenmp conv_direct.c -> libtsm_oracle.so (skipped if up to date)."""
    if (not force and os.path.exists(LIB_PATH)
            and os.path.getmtime(LIB_PATH) >= os.path.getmtime(SRC_PATH)):
        return LIB_PATH
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
           "-o", LIB_PATH, SRC_PATH]
    subprocess.check_call(cmd)
    return LIB_PATH


if __name__ == "__main__":
    print(build(force=True))
