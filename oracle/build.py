"""Compile the CPU oracle (test infrastructure) into oracle/libqg_oracle.so.

Flags matter for bit-exactness of the quantizer: no fast-math, no FMA contraction.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "qg_oracle.c")
OUT_DIR = HERE
OUT = os.path.join(OUT_DIR, "libqg_oracle.so")

FLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC",
         "-shared", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    os.makedirs(OUT_DIR, exist_ok=True)
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    subprocess.run(["gcc", *FLAGS, SRC, "-o", OUT, "-lm"], check=True)
    return OUT


if __name__ == "__main__":
    print(build())
