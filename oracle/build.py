"""Compile the oracle's C source with gcc into ``oracle/liborc_attention.so``.

The same source is compiled twice into one library: accumulators in double (symbols
``*_f64``, used for parity) and in float (symbols ``*_f32``, used to bound fp32 rounding).
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "attention.c")
LIB = os.path.join(HERE, "liborc_attention.so")


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    objs = []
    for acc, suffix in (("double", "f64"), ("float", "f32")):
        obj = os.path.join(HERE, f"attention_{suffix}.o")
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-fopenmp", "-ffp-contract=off",
                               f"-DACC_T={acc}", f"-DSUFFIX={suffix}", "-c", SRC, "-o", obj])
        objs.append(obj)
    subprocess.check_call(["gcc", "-shared", "-fopenmp", "-o", LIB] + objs + ["-lm"])
    for o in objs:
        os.remove(o)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
