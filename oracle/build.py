"""Builds oracle/libmixers_omp.so, the fp64 C / OpenMP twin of the numpy oracle (test infrastructure only).

    python -m oracle.build

Plain gcc, no architecture flags: the library is built here and run on whichever host the tests or the benchmark
use.  -ffp-contract=off keeps every multiply and add a separate fp64 operation, as in the numpy oracle.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libmixers_omp.so")


def build(verbose: bool = False) -> str:
    cmd = [os.environ.get("CC", "gcc"), "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-Wall",
           os.path.join(HERE, "mixers_omp.c"), "-o", LIB, "-lm"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("command failed: %s\n%s\n%s" % (" ".join(cmd), res.stdout, res.stderr))
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
