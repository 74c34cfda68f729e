"""Compiles the oracle's C source with gcc (no GPU, no HIP)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ink_oracle.c")
LIB = os.path.join(HERE, "libink_oracle.so")


def build(force=False):
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        # -mfma: fmaf() becomes the hardware's fused multiply-add (correctly rounded either way);
        # -ffp-contract=off: nothing else is ever fused; no -ffast-math: no sum is re-associated
        subprocess.check_call(["gcc", "-O3", "-mavx2", "-mfma", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC",
                               "-o", LIB, SRC, "-lm"])
    return LIB


if __name__ == "__main__":
    print(build(force=True))
