"""Compile the reference convolutions (oracle/conv_ref.c) into oracle/libconvref.so with gcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libconvref.so")


def build(force=False):
    src = os.path.join(HERE, "conv_ref.c")
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(src):
        return LIB
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-o", LIB, src])
    return LIB


if __name__ == "__main__":
    print(build(force=True))
