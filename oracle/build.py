"""Compile the CPU oracle (test infrastructure) with gcc.

Two shared objects are produced from the one source file: ``libqbo.so`` (serial) and
``libqbo_omp.so`` (the same code with its OpenMP pragmas enabled, used as the timed CPU
baseline).  Floating-point contraction is switched off so that every binary32 step of the
quantizer is a single rounding.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "qbert_oracle.c")
FLAGS = ["-O2", "-ffp-contract=off", "-std=c99", "-Wall", "-Wextra", "-fPIC", "-shared"]


def lib_path(openmp=False):
    return os.path.join(HERE, "libqbo_omp.so" if openmp else "libqbo.so")


def build(force=False):
    for omp in (False, True):
        out = lib_path(omp)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
            continue
        cmd = ["gcc"] + FLAGS + (["-fopenmp"] if omp else []) + [SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build(force=True)
    print("built", lib_path(False), lib_path(True))
