"""Compile the oracle's C layer functions into oracle/liboracle_nn.so (gcc, OpenMP).

TEST INFRASTRUCTURE ONLY.  Plain optimisation flags, no fast-math: every sum
keeps the order written in nn_layers.c.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))


def build(verbose=False):
    src = os.path.join(HERE, "nn_layers.c")
    out = os.path.join(HERE, "liboracle_nn.so")
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", out, src, "-lm"]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
