"""CPU-only tests of the library's host side: it loads, exports what lkv.h declares, and its
allocator / block tables / slot mappings / layer plan agree bit-for-bit with the oracle."""
import os
import re

import numpy as np
import pytest

from oracle import layerkv_oracle as orc
from paper_2410_00428_amd import binding as lkv
from paper_2410_00428_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "lkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lkv_[a-z_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = lkv.load_library()
    names = header_symbols()
    assert len(names) >= 20
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in lkv.h but not exported"
    assert sorted(lkv.EXPORTS) == names


def logical(L=3, Hq=4, Hkv=2, d=64, bs=16, pool=64, dtype="bf16"):
    return lkv.LKV(L, Hq, Hkv, d, bs, pool, dtype, logical_only=True)


def test_create_rejects_bad_configs():
    for kw in (dict(Hq=3, Hkv=2), dict(pool=0), dict(L=0), dict(d=6), dict(bs=0)):
        with pytest.raises(lkv.LkvError) as e:
            logical(**kw)
        assert e.value.status in (lkv.LKV_ERR_INVALID_ARG, lkv.LKV_ERR_UNSUPPORTED)
    with pytest.raises(lkv.LkvError):
        lkv.LKV(1, 1, 1, 64, 16, 8, "bf16", decode_partition=100, logical_only=True)


def test_device_calls_fail_loudly_on_a_logical_context():
    c = logical()
    with pytest.raises(lkv.LkvError) as e:
        c.write_kv(0, 0, 0, 0, 0)
    assert e.value.status == lkv.LKV_ERR_DEVICE
    with pytest.raises(lkv.LkvError):
        c.paged_decode_attention(0, 0, 0, 0, 0, 0, 0)
    for call in (lambda: c.reserve_decode_workspace(4, 64), lambda: c.paged_decode_attention_static(0, 0, 0, 0, 0, 0, 0)):
        with pytest.raises(lkv.LkvError) as e:
            call()
        assert e.value.status == lkv.LKV_ERR_DEVICE
    assert c.layer_residency(0, 0) == lkv.LKV_RES_NONE      # a logical context has no transfers: never IN_FLIGHT


def test_random_op_sequence_matches_oracle_bit_for_bit():
    rng = np.random.default_rng(31)
    L, bs, N = 3, 16, 96
    c = logical(L=L, bs=bs, pool=N)
    o = orc.LayerKVOracle(L, 4, 2, 64, bs, N, "bf16")
    order = rng.permutation(N).astype(np.int32)
    c.pool_reset(order)
    o.pool_reset(order)
    lens = {}
    for step in range(600):
        seq, layer = int(rng.integers(0, 6)), int(rng.integers(0, L))
        op = rng.random()
        key = (seq, layer)
        if op < 0.55:
            n = lens.get(key, 0) + int(rng.integers(0, 70))
            try:
                o.alloc_layer_blocks(seq, layer, n)
                ok = True
            except orc.NoBlocks:
                ok = False
            if ok:
                c.alloc_layer_blocks(seq, layer, n)
                lens[key] = n
            else:
                with pytest.raises(lkv.LkvError) as e:
                    c.alloc_layer_blocks(seq, layer, n)
                assert e.value.status == lkv.LKV_ERR_NO_BLOCKS
        elif op < 0.8 and o.layer_residency(seq, layer) == orc.GPU:
            to_host = bool(rng.random() < 0.5)
            o.free_layer_blocks(seq, layer, to_host=to_host)
            c.free_layer_blocks(seq, layer, to_host)
            if not to_host:
                lens.pop(key, None)
        elif op < 0.85:
            o.free_seq(seq)
            c.free_seq(seq)
            for l in range(L):
                lens.pop((seq, l), None)
        # compare the complete visible state
        assert c.num_free_blocks() == o.num_free_blocks()
        for s in range(6):
            for l in range(L):
                res = o.layer_residency(s, l)
                assert c.layer_residency(s, l) == {None: 0, orc.GPU: 1, orc.HOST: 2}[res]
                if res == orc.HOST:
                    with pytest.raises(lkv.LkvError) as e:
                        c.get_block_table(s, l)
                    assert e.value.status == lkv.LKV_ERR_NOT_RESIDENT
                else:
                    assert c.get_block_table(s, l).tolist() == o.block_table(s, l)
        if o.layer_residency(seq, layer) == orc.GPU and lens.get(key, 0) > 0:
            n = lens[key]
            p0 = int(rng.integers(0, n))
            cnt = int(rng.integers(0, n - p0 + 1))
            assert np.array_equal(c.build_slot_mapping(seq, layer, p0, cnt), o.slot_mapping(seq, layer, p0, cnt))
    c.destroy()


def test_error_codes():
    c = logical(pool=8)
    with pytest.raises(lkv.LkvError) as e:
        c.alloc_layer_blocks(0, 7, 10)
    assert e.value.status == lkv.LKV_ERR_INVALID_ARG
    with pytest.raises(lkv.LkvError) as e:
        c.alloc_layer_blocks(0, 0, 16 * 9)
    assert e.value.status == lkv.LKV_ERR_NO_BLOCKS and c.num_free_blocks() == 8
    with pytest.raises(lkv.LkvError) as e:
        c.build_slot_mapping(0, 0, 0, 4)
    assert e.value.status == lkv.LKV_ERR_NOT_RESIDENT
    c.alloc_layer_blocks(0, 0, 20)
    with pytest.raises(lkv.LkvError) as e:
        c.build_slot_mapping(0, 0, 30, 4)  # beyond the allocated blocks
    assert e.value.status == lkv.LKV_ERR_INVALID_ARG
    with pytest.raises(lkv.LkvError) as e:
        c.free_layer_blocks(1, 0)
    assert e.value.status == lkv.LKV_ERR_NOT_RESIDENT
    with pytest.raises(lkv.LkvError) as e:
        c.pool_reset([0, 1, 2, 3, 4, 5, 6, 6])
    assert e.value.status == lkv.LKV_ERR_INVALID_ARG
    c.destroy()


def test_default_free_order_hands_out_block_zero_first():
    c = logical(pool=8)
    c.alloc_layer_blocks(0, 0, 33)
    assert c.get_block_table(0, 0).tolist() == [0, 1, 2]


def test_plan_retained_layers_matches_paper_example_and_oracle():
    assert lkv.plan_retained_layers(8, 4) == [1, 3, 5, 7]  # Section 3.2.2's example
    for L in (8, 32, 80):
        for x in range(L + 1):
            assert lkv.plan_retained_layers(L, x) == orc.retained_layers(L, x)
    assert tuple(l for l in range(32) if l not in lkv.plan_retained_layers(32, 8)) == wl.OFFLOAD_24_OF_32


def test_fragmenting_schedule_gives_fragmented_identical_tables():
    w = wl.workload(4)
    L, bs = 2, w.shape.block_size
    lens = w.decode_lens
    per_layer = sum(wl.blocks_for(n, bs) for n in lens)
    N = int(per_layer * L * 1.25) + 1024
    c = lkv.LKV(L, 64, 8, 128, bs, N, "bf16", logical_only=True)
    o = orc.LayerKVOracle(L, 64, 8, 128, bs, 1, "bf16")  # tiny data pool: only the logic is used
    o.num_pool_blocks = N
    order = wl.free_list_order(4, N)
    c.pool_reset(order)
    o.pool_reset(order)
    for layer in range(L):
        for op in wl.fragmenting_schedule(4, layer, lens, bs):
            if op.op == "alloc":
                c.alloc_layer_blocks(op.seq, op.layer, op.tokens)
                o.alloc_layer_blocks(op.seq, op.layer, op.tokens)
            else:
                c.free_layer_blocks(op.seq, op.layer)
                o.free_layer_blocks(op.seq, op.layer)
    jumps = total = 0
    for layer in range(L):
        for s, n in enumerate(lens):
            t = c.get_block_table(s, layer)
            assert t.tolist() == o.block_table(s, layer) and len(t) == wl.blocks_for(n, bs)
            jumps += int((np.diff(t) != 1).sum())
            total += len(t) - 1
    assert jumps / total >= 0.5
    assert c.get_block_table(0, 0).tolist() != c.get_block_table(0, 1).tolist()
    c.destroy()


@pytest.mark.parametrize("threads,units", [(3, 3), (1, 1), (4, 2)])
def test_pinned_ring_and_drain_threads_under_a_thread_sanitizer(tmp_path, threads, units):
    """The bounded ring of transfer units and its CPU threads (Section 4), without a GPU: a stand-in copy engine
    fills units, workers drain them into per-layer images; every image complete and exact, every unit handed back
    once, split memcpy exact, a failed wait reported; the build's thread sanitizer must stay silent."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("no host compiler")
    exe = str(tmp_path / "host_tier_test")
    src = os.path.join(ROOT, "tests", "native", "host_tier_test.cpp")
    inc = os.path.join(ROOT, "paper_2410_00428_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-I", inc, src, "-o", exe, "-lpthread"],
                   check=True)
    r = subprocess.run([exe, str(threads), str(units)], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "ThreadSanitizer" not in r.stderr
    assert "host_tier_test: ok" in r.stdout


def test_tier_and_gate_calls_validate_arguments_without_a_device():
    c = logical()
    for call in (lambda: c.host_tier_config(0, 0, 0), lambda: c.host_tier_synchronize(0),
                 lambda: c.offload_layer_pageable(0, [0], np.zeros(8, np.uint8)),
                 lambda: c.reload_layer_pageable(0, [0], np.zeros(8, np.uint8))):
        with pytest.raises(lkv.LkvError) as e:
            call()
        assert e.value.status == lkv.LKV_ERR_DEVICE
    with pytest.raises(lkv.LkvError) as e:
        c.set_link_gate(lambda: False, delay_us=-1)
    assert e.value.status == lkv.LKV_ERR_INVALID_ARG
    c.set_link_gate(lambda: False, delay_us=0, max_checks=3)   # host state only: allowed
    c.set_link_gate(None)


def test_header_is_plain_c_and_the_library_links_and_runs_from_c(tmp_path):
    """include/lkv.h compiles as pedantic C99, and a C program linked against liblkv.so runs the device-free part
    of the ABI (logical context, layer plan, retention driver) to the documented results."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no host compiler")
    exe = str(tmp_path / "c_abi_check")
    libdir = os.path.dirname(lkv.LIB_PATH)
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                        os.path.join(ROOT, "tests", "native", "c_abi_check.c"), "-o", exe, "-L", libdir, "-llkv",
                        "-Wl,-rpath," + libdir], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "c_abi_check: ok" in r.stdout, r.stdout + r.stderr


def test_bench_cuts_the_workload_5_batch_to_the_host_memory_there_is(monkeypatch):
    """The default bench line keeps 211 GiB of layer images in host memory; on a smaller machine it must shrink the
    decode batch (and say so) rather than be killed."""
    import types
    import bench

    def images(n, fp8=False):
        w = wl.workload(5, decode_seqs_cfg5=n)
        blocks = sum(wl.blocks_for(t, w.shape.block_size) for t in w.decode_lens)
        return len(w.offload_layers) * blocks * w.shape.block_bytes // (2 if fp8 else 1)

    monkeypatch.setattr(bench, "host_memory_available", lambda: 1 << 62)
    assert bench.fit_decode_seqs(types.SimpleNamespace(decode_seqs=64, kv_dtype="bf16")) == 64
    monkeypatch.setattr(bench, "host_memory_available", lambda: 270 << 30)
    assert bench.fit_decode_seqs(types.SimpleNamespace(decode_seqs=64, kv_dtype="bf16")) == 64
    assert images(64) + (24 << 30) <= 270 << 30
    for avail_gib in (200, 100, 40):
        monkeypatch.setattr(bench, "host_memory_available", lambda a=avail_gib: a << 30)
        n = bench.fit_decode_seqs(types.SimpleNamespace(decode_seqs=64, kv_dtype="bf16"))
        assert 4 <= n < 64 and n % 4 == 0
        assert images(n) + (24 << 30) <= avail_gib << 30 or n == 4
        assert images(n + 4) + (24 << 30) > avail_gib << 30
    monkeypatch.setattr(bench, "host_memory_available", lambda: 150 << 30)
    assert bench.fit_decode_seqs(types.SimpleNamespace(decode_seqs=64, kv_dtype="fp8")) == 64   # half-size images
    assert bench.host_memory_available() > 0
