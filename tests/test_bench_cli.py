"""bench.py without a GPU: the one-GPU rule, the flop count the TFLOP/s figures are built on, and that the
orchestration modules import (they only touch the device when an engine is constructed)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="4")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_causal_flops_of_the_workloads():
    """4 d Hq sum n(n+1)/2 per layer: 2.75e11 for 8 x 2048, 8.80e12 for 4 x 16384, 1.10e12 for 2 x 8192 tokens at
    32 heads of 128 channels (the figures the scope table of this build quotes)."""
    import bench
    from paper_2410_00428_amd import workloads as wl
    for number, want in ((2, 2.75e11), (3, 8.80e12), (5, 1.10e12)):
        w = wl.workload(number)
        got = bench.causal_flops(w.prompt_lens, w.shape.num_q_heads, w.shape.head_dim)
        assert abs(got - want) / want < 5e-3, (number, got)
    assert bench.causal_flops([1], 1, 1) == 4.0          # one query, one key: one product and one weighted value
    assert bench.causal_flops([3], 2, 8) == 4.0 * 8 * 2 * 6


def test_orchestration_modules_import_without_a_device():
    pytest.importorskip("torch")
    from paper_2410_00428_amd import engine, serving  # noqa: F401
    assert hasattr(engine, "LayerKVEngine") and hasattr(serving, "MixedIteration")
