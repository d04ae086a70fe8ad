"""Compile the C part of the oracle (test infrastructure): python -m oracle.build -> oracle/liboracle_fast.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "liboracle_fast.so")


def build(verbose=True):
    src = os.path.join(HERE, "csrc", "perturb_fast.c")
    # -ffp-contract=off: the formula's inner products are rounded to fp32 before its one fused step
    cmd = [os.environ.get("CC", "gcc"), "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-std=c11", src,
           "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
