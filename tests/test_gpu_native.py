"""The C ABI used from a C++ program with plain HIP memory (no Python, no torch): ``tests/native/gpu_consumer.cpp``
runs one layer through write, prefill, offload, reload and decode and checks the results against a dense
double-precision attention of its own.  The program is built by ``__graft_entry__.build()``; this test runs it."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "native", "_build", "gpu_consumer")


def test_cxx_consumer_of_the_c_abi_runs_the_path_without_python_memory():
    assert os.path.exists(EXE), "tests/native/_build/gpu_consumer is not built: run __graft_entry__.build() first"
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, f"exit {r.returncode}\n{r.stdout}\n{r.stderr}"
    assert "gpu_consumer: ok" in r.stdout
