"""Compile the oracle's C convolution (gcc, OpenMP) into oracle/liboracle_conv.so.

TEST INFRASTRUCTURE ONLY.  Building the checker is not using it: the product's
build step may call this, the product path never loads the result.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "conv_direct.c")
LIB = os.path.join(HERE, "liboracle_conv.so")


def build(force=False):
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c11",
           "-Wall", "-o", LIB, SRC]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
