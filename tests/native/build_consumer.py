"""Builds ``tests/native/gpu_consumer.cpp`` (a C++ program that uses the C ABI with plain HIP memory) against the
in-tree library into ``tests/native/_build/gpu_consumer``.  Called by ``__graft_entry__.build()``; the GPU test only
runs the result."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
EXE = os.path.join(HERE, "_build", "gpu_consumer")


def build() -> str:
    from paper_2410_00428_amd.build import _hipcc
    lib_dir = os.path.join(ROOT, "paper_2410_00428_amd")
    os.makedirs(os.path.dirname(EXE), exist_ok=True)
    # host code only (no kernels of its own); the library is found next to the package at run time
    cmd = [_hipcc(), "-std=c++17", "-O1", "-Wall", "-I" + os.path.join(ROOT, "include"),
           os.path.join(HERE, "gpu_consumer.cpp"), "-L" + lib_dir, "-llkv",
           "-Wl,-rpath," + os.path.join("$ORIGIN", "..", "..", "..", "paper_2410_00428_amd"), "-o", EXE]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError(f"{' '.join(cmd)}\n{r.stdout}\n{r.stderr}")
    return EXE


if __name__ == "__main__":
    print(build())
