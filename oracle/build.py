"""Compile the CPU oracle (plain C, gcc) into oracle/liboracle.so.

TEST INFRASTRUCTURE ONLY -- see direct_conv.c.  No -march=native: the built
library travels to other machines.  No -ffast-math and no FMA contraction:
the oracle's arithmetic is exactly the double operations written in the source.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "liboracle.so")


def build(verbose: bool = False) -> str:
    cmd = ["gcc", "-O3", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
           "-Wall", "-o", LIB, os.path.join(HERE, "direct_conv.c")]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
