"""Compiles the CPU oracle (test infrastructure) into shared libraries beside this file.

    python oracle/build.py

Two builds of the same source: `libhet_oracle.so` computes in double (the oracle used for
parity), `libhet_oracle_f32.so` in float (used only to show how far single-precision rounding
alone moves the values).  Contraction is off so every operation rounds once.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "het_oracle.c")
FLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-Wall", "-Wextra"]


def build(verbose: bool = False) -> None:
    for name, real in (("libhet_oracle.so", "double"), ("libhet_oracle_f32.so", "float")):
        cmd = ["gcc", *FLAGS, f"-DHET_REAL={real}", SRC, "-o", os.path.join(HERE, name), "-lm"]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
