"""Compiles the oracle's plain C routines with gcc (test infrastructure only)."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))


def build():
    src = os.path.join(_HERE, "orc_kernels.c")
    out = os.path.join(_HERE, "liborc.so")
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", out, src])
    return out


if __name__ == "__main__":
    print(build())
