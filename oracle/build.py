"""Compile the CPU oracle (plain C++17) into oracle/liblpco.so.

Test infrastructure only: the product library never links or loads this.
Usage: python oracle/build.py
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ["lpco_philox.cpp", "lpco_quant.cpp", "lpco_glm.cpp", "lpco_mlp.cpp", "lpco_svrg.cpp"]
OUT = os.path.join(HERE, "liblpco.so")


def build(verbose=False):
    cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-fopenmp",
           # the quantizer's float arithmetic decides integer codes: no fused
           # multiply-add contraction, no value-changing optimisation
           "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", "-o", OUT] + [os.path.join(HERE, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True, cwd=HERE)
    return OUT


def needs_build():
    if not os.path.exists(OUT):
        return True
    t = os.path.getmtime(OUT)
    deps = SOURCES + ["lpco.h"]
    return any(os.path.getmtime(os.path.join(HERE, s)) > t for s in deps)


if __name__ == "__main__":
    build(verbose=True)
    print("built", OUT)
    sys.exit(0)
