"""TEST INFRASTRUCTURE ONLY -- compiles the oracle's C convolution loops with gcc.

Running `python -m oracle.build` (or calling `build()`) produces
`oracle/liboracle_conv.so` next to the source.  The GPU library is not involved.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "conv_direct.c")
LIB = os.path.join(HERE, "liboracle_conv.so")


def build(force: bool = False) -> str:
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", LIB, SRC]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
