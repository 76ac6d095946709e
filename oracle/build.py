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


def build_sanitized():
    """The same loops under AddressSanitizer and UndefinedBehaviorSanitizer (no -O3), linked with the
    driver oracle/sanitize_check.c into the executable oracle/sanitize_check: run it, exit status 0 =
    no out-of-bounds access, no undefined behaviour, adjoint identities hold."""
    exe = os.path.join(HERE, "sanitize_check")
    cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-fopenmp", "-std=c11", "-Wall", "-Wextra", "-o", exe,
           os.path.join(HERE, "sanitize_check.c"), SRC, "-lm"]
    subprocess.check_call(cmd)
    return exe


if __name__ == "__main__":
    import sys
    print(build_sanitized() if "--sanitize" in sys.argv else build(force=True))
