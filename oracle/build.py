"""Compile the CPU oracle (test infrastructure) into oracle/libcombo_ref.so.

Plain g++ -O2, no OpenMP, no -march flags, floating-point contraction off so that
every product and sum is rounded on its own as the oracle's comments state.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "combo_ref.cpp")
LIB = os.path.join(HERE, "libcombo_ref.so")

FLAGS = ["-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
         "-Wall", "-Wextra"]


def build(verbose=False):
    cmd = ["g++"] + FLAGS + ["-o", LIB, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
