"""Builds the C oracle (oracle/mbq_oracle.c) into oracle/libmbq_oracle.so with gcc; test and benchmark
infrastructure only, never linked into the HIP library.  Run: python -m oracle.build"""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "mbq_oracle.c")
LIB = os.path.join(HERE, "libmbq_oracle.so")


def build() -> str:
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        raise RuntimeError("no C compiler found for the C oracle")
    # -O2, IEEE arithmetic as written: no fast-math, no contraction of a*b+c into fused operations
    cmd = [cc, "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", "-o", LIB, SRC, "-lm"]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), proc.stdout))
    return LIB


if __name__ == "__main__":
    print("built", build())
