"""Compile the CPU oracle (plain C99, gcc) into oracle/libbdr_ref.so.

Test infrastructure only: nothing in the product path may call this library.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libbdr_ref.so")


def build(verbose: bool = False) -> str:
    cmd = [
        "gcc", "-std=c99", "-O2", "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra",
        "-shared", "-fPIC", "-o", LIB, os.path.join(HERE, "bdr_ref.c"), "-lm",
    ]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
