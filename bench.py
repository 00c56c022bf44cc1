#!/usr/bin/env python3
"""Benchmark of the layer-wise paged KV cache hot path on one MI355X.

Default: workload 5, the largest configuration that runs on one GPU (LLaMA-2-7B KV shape, bf16): one "step" is one
mixed serving iteration at full size (see mixed_iteration below): 64 decoding sequences whose 24 host-resident
layers are reloaded through a ring of blocks, paged decode attention of every layer, and two new 8192-token prompts
that are written, attended (causal prefill) and offloaded in the same iteration.  The same line carries, as named
components, a full step of workload 3 (4 prompts x 16384 tokens: write, causal prefill, 24 layers offloaded and
reloaded, 64 decode steps) and of workload 2 (8 x 2048, 16 layers offloaded and reloaded, one decode step), each
with its own short warm-up and step count.  Inputs are resident in HBM before a timed region starts.  Prints ONE
JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 5|3|2] [--no-components] [--no-cpu-baseline]

--workload 2 / 3 time that workload's step alone (allocate + map, write K/V, causal prefill attention, pack + copy
of the offloaded layers on a side stream, reload, decode steps) with all of its extra measurements.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.md")


def measured_traffic(kernel: str, workload: int):
    """HBM bytes per launch of `kernel` at `workload` as two rocprofv3 --pmc runs counted them (FETCH_SIZE, then
    WRITE_SIZE, each scaled by what the same counter reads for a copy kernel of known size).  The one place these
    figures live is the table of profiles/hbm_traffic.md (rows `| kernel | workload | fetched bytes | written bytes
    | ...`), which also gives the commands and the scale factors; None when the table has no such row."""
    try:
        rows = open(TRAFFIC_FILE).read().splitlines()
    except OSError:
        return None
    for line in rows:
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 4 and cells[0] == kernel and cells[1] == str(workload):
            try:
                return float(cells[2]) + float(cells[3])
            except ValueError:
                return None
    return None

METRIC = "decode paged-attn HBM GB/s; prefill attn TFLOP/s; layer offload/reload GB/s"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", type=int, default=5, choices=(2, 3, 5),
                    help="5 (default, the largest single-GPU configuration): the mixed serving iteration with the "
                         "decode batch's host layers in ordinary host memory (needs ~215 GiB of host memory at 64 "
                         "decode sequences), with a step of workloads 3 and 2 as components; 2 or 3: that workload alone")
    ap.add_argument("--no-components", action="store_true",
                    help="workload 5 only: skip the steps of workloads 3 and 2 that the line carries as components")
    ap.add_argument("--component", action="store_true",
                    help="workloads 2 and 3: print the cut of the figures that the default line carries for them (what "
                         "the default run asks of its child processes)")
    ap.add_argument("--component-steps", type=int, default=0,
                    help="timed steps of the workload 3 / workload 2 components (0: 2 resp. 5)")
    ap.add_argument("--decode-seqs", type=int, default=64, help="workload 5: decoding sequences (64 = the full size)")
    ap.add_argument("--ring-layers", type=int, default=3, help="workload 5: sets of blocks the host layers pass through")
    ap.add_argument("--tier-unit-mib", type=int, default=64, help="workload 5: size of one unit of the pinned ring")
    ap.add_argument("--tier-units", type=int, default=4, help="workload 5: units in the pinned ring")
    ap.add_argument("--tier-threads", type=int, default=8,
                    help="workload 5: CPU threads that copy between the pinned ring and ordinary host memory")
    ap.add_argument("--kv-dtype", default="bf16", choices=("bf16", "fp8"),
                    help="fp8: the same step over an 8-bit pool (E4M3 codes); not the headline configuration")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-offload", action="store_true",
                    help="keep every layer on the GPU: a step without host-link traffic (profiling runs: under "
                         "rocprofv3 copies run as shader kernels and slow the kernels next to them)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the figures of the other workloads' decode batches and of the 8-bit pool (profiling runs)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget for the oracle timing")
    return ap.parse_args()


def causal_flops(lens, Hq, d):
    return 4.0 * d * Hq * sum(n * (n + 1) / 2 for n in lens)


def cpu_baseline(w, seconds: float, lens=None) -> dict:
    """The oracle as it stands, timed on the host: paged decode attention of ONE layer of the
    workload (all sequences unless `lens` names a sample of them, all heads, fp64 accumulators), repeated until
    ~`seconds` are spent."""
    from oracle import layerkv_oracle as orc
    from paper_2410_00428_amd import workloads as wl
    sh = w.shape
    lens = list(lens) if lens is not None else [n + 1 for n in w.prompt_lens]
    nblk = sum(wl.blocks_for(n, sh.block_size) for n in lens)
    o = orc.LayerKVOracle(1, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.block_size, nblk, sh.dtype)
    o.pool_reset(wl.free_list_order(w.number, nblk, index=77))
    rng = np.random.default_rng(wl.SEED_BASE + w.number)
    # fill the blocks directly with seeded bf16 values (the oracle's own write path is not what is timed)
    o.pool[:] = wl.normal_tensor(rng, o.pool.shape, w.data_scale, sh.dtype)
    for s, n in enumerate(lens):
        o.alloc_layer_blocks(s, 0, n)
    q = wl.normal_tensor(rng, (len(lens), sh.num_q_heads, sh.head_dim), w.data_scale, sh.dtype)
    bt = o.padded_block_table(range(len(lens)), 0)
    threads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1))
    kv_bytes = sum(lens) * sh.token_bytes
    o.paged_decode_attention(q, bt, lens, threads=threads)  # warm
    reps, t0 = 0, time.perf_counter()
    while True:
        o.paged_decode_attention(q, bt, lens, threads=threads)
        reps += 1
        el = time.perf_counter() - t0
        if el > seconds:
            break
    t1 = time.perf_counter()
    o.paged_decode_attention(q, bt, lens, threads=1)
    decode_1core = kv_bytes / (time.perf_counter() - t1) / 1e9
    # the byte movers of the same layer: write of every token's K/V, gather of the layer's blocks, scatter back
    ids = sum((o.block_table(s, 0) for s in range(len(lens))), [])
    slots = np.concatenate([o.slot_mapping(s, 0, 0, n) for s, n in enumerate(lens)])
    Kw, Vw = (wl.normal_tensor(rng, (sum(lens), sh.num_kv_heads, sh.head_dim), w.data_scale, sh.dtype) for _ in range(2))
    t1 = time.perf_counter()
    o.write_kv(Kw, Vw, slots)
    t_write = time.perf_counter() - t1
    t1 = time.perf_counter()
    image = o.pack_layer_blocks(ids)
    t_pack = time.perf_counter() - t1
    t1 = time.perf_counter()
    o.unpack_layer_blocks(ids, image)
    t_unpack = time.perf_counter() - t1
    movers = {"decode_GBps_1_core": round(decode_1core, 3),
              "write_kv_GBps": round(2 * kv_bytes / t_write / 1e9, 3),
              "pack_GBps": round(2 * len(ids) * sh.block_bytes / t_pack / 1e9, 3),
              "unpack_GBps": round(2 * len(ids) * sh.block_bytes / t_unpack / 1e9, 3),
              "movers_note": "oracle write / pack / unpack of the same layer, bytes read + written, one call each, "
                             "single-threaded numpy"}
    del Kw, Vw, image
    # a second figure for the contraction: causal prefill on a seeded sample of query rows
    T = sum(w.prompt_lens)
    n0 = w.prompt_lens[0]
    Q1, K1, V1 = (wl.normal_tensor(rng, (n0, h, sh.head_dim), w.data_scale, sh.dtype)
                  for h in (sh.num_q_heads, sh.num_kv_heads, sh.num_kv_heads))
    # about a tenth of the layer's causal flops: every head, a seeded sample of rows (a few seconds on 16 cores)
    rows = wl.sample_rows(rng, n0, min(n0, 1024))
    tok = np.repeat(rows, sh.num_q_heads)
    head = np.tile(np.arange(sh.num_q_heads, dtype=np.int32), len(rows))
    t1 = time.perf_counter()
    orc.prefill_attention_rows(Q1, K1, V1, [0, n0], sh.dtype, tok, head, threads=threads)
    t_rows = time.perf_counter() - t1
    flops_rows = float(sum(4.0 * sh.head_dim * (r + 1) for r in tok))
    return {"value": round(kv_bytes * reps / el / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"paged decode attention of one layer of workload {w.number} ({len(lens)} seqs x "
                      f"{sh.num_q_heads} heads, contexts {min(lens)}..{max(lens)}, {kv_bytes / 2**20:.0f} MiB KV), fp64 accumulators, "
                      f"{reps} repetitions in {el:.1f} s",
            "prefill_tflops": round(flops_rows / t_rows / 1e12, 6),
            "prefill_sample": f"{len(rows)} sampled causal rows x {sh.num_q_heads} heads of one {n0}-token prompt "
                              f"({flops_rows:.3g} flop in {t_rows:.1f} s)", **movers}


def decode_other_workloads(torch, dev, numbers=(3, 4, 5)) -> dict:
    """Paged decode attention of the other configurations' decode batches (not bench lines: context for the
    headline figure).  A few layers of the workload's KV, blocks handed out in a seeded random order over the pool,
    the layers taken in turn so that nothing stays in the last-level cache; kernel time from the library's events."""
    from paper_2410_00428_amd import binding as lkv_b
    from paper_2410_00428_amd import workloads as wl
    out = {}
    for number, layers in ((3, 8), (4, 16), (5, 2)):
        if number not in numbers:
            continue
        w = wl.workload(number)
        sh = w.shape
        lens = [n + 1 for n in w.prompt_lens] if number == 3 else list(w.decode_lens)
        B = len(lens)
        nblk = sum(wl.blocks_for(n, sh.block_size) for n in lens) * layers
        pool = (torch.randn(nblk * sh.block_bytes // 2, device=dev, dtype=torch.float32) * w.data_scale).to(torch.bfloat16)
        c = lkv_b.LKV(layers, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.block_size, nblk, "bf16", pool=pool)
        c.pool_reset(wl.free_list_order(number, nblk, index=55))
        tables = []
        for l in range(layers):
            for s_, n in enumerate(lens):
                c.alloc_layer_blocks(s_, l, n)
            tables.append(torch.from_numpy(c.padded_block_table(range(B), l)).to(dev))
        cl = torch.tensor(lens, dtype=torch.int32, device=dev)
        q = (torch.randn(B, sh.num_q_heads, sh.head_dim, device=dev) * w.data_scale).to(torch.bfloat16)
        o = torch.empty_like(q)
        reps = 3

        def sweep():
            for l in range(layers):
                c.paged_decode_attention(l, q, o, tables[l], tables[l].shape[1], cl, B)
        sweep()
        torch.cuda.synchronize()
        c.set_profiling(True)
        s0 = c.get_stats()
        for _ in range(reps):
            sweep()
        s1 = c.get_stats()
        c.set_profiling(False)
        us = (s1["decode_kernel_ns"] - s0["decode_kernel_ns"]) / (reps * layers) * 1e-3
        kv_bytes = sum(lens) * sh.token_bytes
        out[str(number)] = {"workload": w.name, "seqs": B, "kv_MiB_per_layer": round(kv_bytes / 2**20, 1),
                            "us_per_layer": round(us, 1), "GBps": round(kv_bytes / us / 1e3, 1),
                            "frac_of_hbm_peak": round(kv_bytes / us / 1e3 / HBM_PEAK_GBS, 4)}
        c.destroy()
        del pool, tables
    return out


def fp8_pool_figures(torch, dev) -> dict:
    """The 8-bit pool (E4M3 codes, the paper's future-work direction) on workload 2's shape: write of 16384 prompt
    tokens per layer and decode attention over 8 x 2049 tokens, 16 layers taken in turn; bytes are the pool's."""
    from paper_2410_00428_amd import binding as lkv_b
    from paper_2410_00428_amd import workloads as wl
    w = wl.workload(2)
    sh = w.shape
    layers, lens = 16, [n + 1 for n in w.prompt_lens]
    B, T = len(lens), sum(w.prompt_lens)
    nblk = sum(wl.blocks_for(n, sh.block_size) for n in lens) * layers
    c = lkv_b.LKV(layers, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.block_size, nblk, "fp8",
                  k_scale=w.data_scale / 16, v_scale=w.data_scale / 16)
    c.pool_reset(wl.free_list_order(2, nblk, index=56))
    slots, tables = [], []
    for l in range(layers):
        for s_, n in enumerate(lens):
            c.alloc_layer_blocks(s_, l, n)
        slots.append(torch.from_numpy(np.concatenate(
            [c.build_slot_mapping(s_, l, 0, n - 1) for s_, n in enumerate(lens)])).to(dev))
        tables.append(torch.from_numpy(c.padded_block_table(range(B), l)).to(dev))
    K = [(torch.randn(T, sh.num_kv_heads, sh.head_dim, device=dev) * w.data_scale).to(torch.bfloat16) for _ in range(4)]
    q = (torch.randn(B, sh.num_q_heads, sh.head_dim, device=dev) * w.data_scale).to(torch.bfloat16)
    o = torch.empty_like(q)
    cl = torch.tensor(lens, dtype=torch.int32, device=dev)

    def sweep():
        for l in range(layers):
            c.write_kv(l, K[l % 4], K[(l + 1) % 4], slots[l], T)
        for l in range(layers):
            c.paged_decode_attention(l, q, o, tables[l], tables[l].shape[1], cl, B)
    sweep()
    torch.cuda.synchronize()
    c.set_profiling(True)
    s0 = c.get_stats()
    for _ in range(3):
        sweep()
    s1 = c.get_stats()
    c.set_profiling(False)
    n_launch = 3 * layers
    dec_us = (s1["decode_kernel_ns"] - s0["decode_kernel_ns"]) / n_launch * 1e-3
    wr_us = (s1["write_kernel_ns"] - s0["write_kernel_ns"]) / n_launch * 1e-3
    kv_bytes = sum(lens) * c.token_bytes
    out = {"pool_bytes_per_token_per_layer": c.token_bytes,
           "decode_us_per_layer": round(dec_us, 1), "decode_pool_GBps": round(kv_bytes / dec_us / 1e3, 1),
           "decode_tokens_per_us": round(sum(lens) / dec_us, 1),
           "write_us_per_layer": round(wr_us, 1),
           "write_GBps_in_plus_out": round(T * (sh.num_kv_heads * sh.head_dim * 2 * 2 + c.token_bytes) / wr_us / 1e3, 1),
           "note": "an offload image is half the bf16 one, so the link time of every offload and reload halves"}
    c.destroy()
    return out


def pinned_copy_peak(torch, dev) -> dict:
    """What one large hipMemcpyAsync between pinned host memory and the device reaches, per direction (GB/s)."""
    def ev():
        return torch.cuda.Event(enable_timing=True)
    link = {}
    big = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    big_host = torch.empty(1 << 30, dtype=torch.uint8, pin_memory=True)
    for name, dst, src in (("d2h", big_host, big), ("h2d", big, big_host)):
        dst.copy_(src, non_blocking=True)
        a, b = ev(), ev()
        a.record()
        for _ in range(2):
            dst.copy_(src, non_blocking=True)
        b.record()
        torch.cuda.synchronize()
        link[name] = 2 * (1 << 30) / (a.elapsed_time(b) * 1e-3) / 1e9
    return link


def host_memory_available() -> int:
    """Bytes of host memory this process may still take: the smaller of the machine's MemAvailable and the room
    left under the memory limit of its control group, when there is one."""
    avail = None
    try:
        for ln in open("/proc/meminfo"):
            if ln.startswith("MemAvailable:"):
                avail = int(ln.split()[1]) * 1024
    except OSError:
        pass
    for lim, cur in (("/sys/fs/cgroup/memory.max", "/sys/fs/cgroup/memory.current"),
                     ("/sys/fs/cgroup/memory/memory.limit_in_bytes", "/sys/fs/cgroup/memory/memory.usage_in_bytes")):
        try:
            a, b = open(lim).read().strip(), open(cur).read().strip()
            if a.isdigit() and int(a) < (1 << 60):
                room = int(a) - int(b)
                avail = room if avail is None else min(avail, room)
        except OSError:
            pass
    return avail if avail is not None else 1 << 62


def fit_decode_seqs(args) -> int:
    """Workload 5 keeps 24 of 32 layers of its decode batch in ordinary host memory (211 GiB at 64 sequences).  On a
    machine that cannot hold that, the batch is cut to the largest number of sequences whose images fit (with 24 GiB
    left for everything else); the line then says so in `config.workload`."""
    from paper_2410_00428_amd import workloads as wl
    asked, avail = args.decode_seqs, host_memory_available()
    n = asked
    while n > 4:
        w = wl.workload(5, decode_seqs_cfg5=n)
        blocks = sum(wl.blocks_for(t, w.shape.block_size) for t in w.decode_lens)
        per_block = w.shape.block_bytes // (2 if args.kv_dtype == "fp8" else 1)
        if len(w.offload_layers) * blocks * per_block + (24 << 30) <= avail:
            break
        n -= 4
    if n != asked:
        print(f"[bench workload 5] host memory available {avail / 2**30:.0f} GiB: decode batch cut from {asked} to {n} "
              f"sequences", file=sys.stderr, flush=True)
    return n


def mixed_iteration(args) -> dict:
    """Workload 5 at its full size: 64 decoding sequences (contexts uniform in [128, 16384], ~8 GiB of KV per
    layer) of which 24 of 32 layers live in ORDINARY host memory (~194 GiB) and come back through a ring of
    blocks, plus two new 8192-token prompts that prefill and offload in the same iteration.  One step = one such
    iteration over all layers.  The iteration is bound by the host link by construction (the paper's extreme
    case); `value` is still the decode kernel's rate, by the library's events inside the iteration."""
    import torch
    from paper_2410_00428_amd import workloads as wl
    from paper_2410_00428_amd.serving import MixedIteration

    def say(msg):
        print(f"[bench workload 5] {msg}", file=sys.stderr, flush=True)

    asked_seqs = args.decode_seqs
    args.decode_seqs = fit_decode_seqs(args)
    w = wl.workload(5, decode_seqs_cfg5=args.decode_seqs)
    kw = {}
    if args.kv_dtype == "fp8":   # the same iteration over an 8-bit pool: every image and every reload is half as large
        import dataclasses
        w = dataclasses.replace(w, shape=dataclasses.replace(w.shape, dtype="fp8"), name=w.name + "-fp8pool")
        kw = dict(k_scale=w.data_scale / 16, v_scale=w.data_scale / 16)
        args.no_cpu_baseline = True   # the timed oracle sample is the bf16 one
    sh = w.shape
    L, bs = sh.num_layers, sh.block_size
    dlens, plens, host = list(w.decode_lens), list(w.prompt_lens), list(w.offload_layers)
    B, Td, T = len(dlens), sum(dlens), sum(plens)
    dblk = sum(wl.blocks_for(n, bs) for n in dlens)
    pblk = sum(wl.blocks_for(n, bs) for n in plens)
    R = args.ring_layers
    nblk = (L - len(host) + R) * dblk + L * pblk + 64
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    say(f"{B} decode sequences, {Td} cached tokens per layer = {dblk * sh.block_bytes / 2**30:.2f} GiB per layer; "
        f"pool {nblk} blocks = {nblk * sh.block_bytes / 2**30:.1f} GiB; host images "
        f"{len(host) * dblk * sh.block_bytes / 2**30:.1f} GiB")
    it = MixedIteration(sh, dlens, plens, host, nblk, ring_layers=R, free_order=wl.free_list_order(5, nblk),
                        tier_unit_bytes=args.tier_unit_mib << 20, tier_units=args.tier_units,
                        tier_threads=args.tier_threads, **kw)
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.SEED_BASE + 5)

    def randn(n, h):   # in pieces: the fp32 draw of a 4 GiB tensor would need 8 GiB more
        out = torch.empty(n, h, sh.head_dim, dtype=torch.bfloat16, device=dev)
        for a in range(0, n, 1 << 16):
            b = min(n, a + (1 << 16))
            out[a:b] = torch.randn(b - a, h, sh.head_dim, generator=gen, device=dev) * w.data_scale
        return out

    Kd, Vd = randn(Td, sh.num_kv_heads), randn(Td, sh.num_kv_heads)
    # queries scaled so that the softmax is neither uniform nor one-hot at these context lengths
    q_dec = [randn(B, sh.num_q_heads) * 0.25 for _ in range(L)]
    O_ref = torch.zeros(L, B, sh.num_q_heads, sh.head_dim, dtype=torch.bfloat16, device=dev)
    O_dec = torch.zeros_like(O_ref)
    n_in = 4
    pq = [(randn(T, sh.num_q_heads) * 0.25, randn(T, sh.num_kv_heads), randn(T, sh.num_kv_heads)) for _ in range(n_in)]
    O_pf = torch.empty_like(pq[0][0])
    t0 = time.perf_counter()
    # layers alternate between the two tensors' roles so that neighbouring layers hold different bytes
    it.build_cached_state(lambda l: (Kd, Vd) if l % 2 == 0 else (Vd, Kd),
                          while_resident=lambda l: it.decode_layer(l, q_dec[l], O_ref[l]),
                          progress=lambda m: say(f"{m} ({time.perf_counter() - t0:.1f} s)"))
    torch.cuda.synchronize()
    t_build = time.perf_counter() - t0
    del Kd, Vd

    def iteration():
        it.run(q_dec, O_dec, lambda l: pq[l % n_in], O_pf)
        it.finish()
        it.drop_prompts()

    for i in range(args.warmup):
        t1 = time.perf_counter()
        iteration()
        say(f"warm-up iteration {i}: {time.perf_counter() - t1:.3f} s")
    exact = bool(torch.equal(O_dec, O_ref)) if args.warmup else None
    it.ctx.set_profiling(True)
    s0 = it.ctx.get_stats()
    walls = []
    for i in range(args.steps):
        O_dec.zero_()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        iteration()
        walls.append(time.perf_counter() - t1)
        say(f"iteration {i}: {walls[-1]:.3f} s")
        exact = bool(torch.equal(O_dec, O_ref)) and exact is not False
    st = it.ctx.get_stats()
    it.ctx.set_profiling(False)
    K = args.steps
    d = {k: st[k] - s0[k] for k in st if isinstance(st[k], int)}
    wall = sum(walls) / K
    kv_bytes = Td * sh.token_bytes
    decode_gbs = kv_bytes * L * K / max(d["decode_kernel_ns"], 1)
    assert d["decode_kernel_launches"] == L * K and d["prefill_kernel_launches"] == L * K
    pf_flops = causal_flops(plens, sh.num_q_heads, sh.head_dim)
    prefill_tflops = pf_flops * L * K / max(d["prefill_kernel_ns"], 1) / 1e3
    reload_bytes = len(host) * dblk * sh.block_bytes
    offload_bytes = len(host) * pblk * sh.block_bytes

    link = pinned_copy_peak(torch, dev)
    reload_gbs = reload_bytes / wall / 1e9
    out = {
        "metric": METRIC, "value": round(decode_gbs, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": round(wall * 1e3, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "kv_pool": sh.dtype,
        "config": {"workload": f"5: {w.name} (L={L}, Hq={sh.num_q_heads}, Hkv={sh.num_kv_heads}, d={sh.head_dim}, block 16, "
                               f"{B} decoding sequences with contexts {min(dlens)}..{max(dlens)} ({Td} tokens), "
                               f"{len(host)} of {L} layers of them in ordinary host memory and reloaded through a ring of "
                               f"{R} sets of blocks, {len(plens)} new prompts x {plens[0]} tokens prefilled and offloaded "
                               f"in the same iteration)"
                               + (f"; DEVIATION: the decode batch is cut from {asked_seqs} sequences because the host "
                                  f"memory of this machine cannot hold their images" if B != asked_seqs else ""),
                   "value_is": "decode paged attention: context KV bytes / HIP-event time of the decode launches "
                               "(library events), measured inside the iteration"},
        "components": {
            "decode_paged_attn_GBps": round(decode_gbs, 2),
            "decode_frac_of_hbm_peak": round(decode_gbs / HBM_PEAK_GBS, 4),
            "decode_ms_per_layer": round(d["decode_kernel_ns"] * 1e-6 / (L * K), 4),
            "prefill_attn_TFLOPs": round(prefill_tflops, 2),
            "prefill_frac_of_bf16_mfma_peak": round(prefill_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
            "prefill_ms_per_layer": round(d["prefill_kernel_ns"] * 1e-6 / (L * K), 4),
            "write_kv_GBps": round(d["write_kernel_bytes"] / max(d["write_kernel_ns"], 1), 2),
            "pack_kernel_GBps": round(d["pack_kernel_bytes"] / max(d["pack_kernel_ns"], 1), 2),
            "unpack_kernel_GBps": round(d["unpack_kernel_bytes"] / max(d["unpack_kernel_ns"], 1), 2),
            "reload_GiB_per_iteration": round(reload_bytes / 2**30, 2),
            "offload_GiB_per_iteration": round(offload_bytes / 2**30, 2),
            "reload_GBps_over_the_iteration": round(reload_gbs, 2),
            "pinned_copy_peak_GBps": {k: round(v, 2) for k, v in link.items()},
            "reload_frac_of_link_peak": round(reload_gbs / link["h2d"], 4),
            "gpu_kernel_ms_per_iteration": round((d["decode_kernel_ns"] + d["prefill_kernel_ns"] + d["write_kernel_ns"]
                                                  + d["pack_kernel_ns"] + d["unpack_kernel_ns"]) * 1e-6 / K, 2),
            "iteration_s": [round(x, 3) for x in walls],
        },
        "memory": {"pool_GiB": round(nblk * sh.block_bytes / 2**30, 1),
                   "host_images_GiB": round((reload_bytes + offload_bytes) / 2**30, 1),
                   "pinned_MiB": args.tier_units * args.tier_unit_mib, "tier_threads": args.tier_threads, "build_cached_state_s": round(t_build, 1)},
        "decode_after_reload_equals_decode_before_offload": exact,
        "roofline": {"kernel": "paged_decode_mfma_kernel (lkv_paged_decode_attention)", "bound": "hbm",
                     "achieved": round(decode_gbs, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(decode_gbs / HBM_PEAK_GBS, 4), "traffic": None,
                     "launch_ms": round(d["decode_kernel_ns"] * 1e-6 / (L * K), 4), "bytes_per_launch": kv_bytes},
    }
    it.close()
    del it, O_ref, O_dec, q_dec, pq, O_pf
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    # the counters were read at the full batch of 64 sequences
    out["roofline"]["traffic"] = (measured_traffic("paged_decode_mfma_kernel", 5)
                                  if args.kv_dtype == "bf16" and B == 64 else None)
    if not args.no_extras:
        # the decode batches of the other configurations (the 70B-shaped GQA batch of workload 4 among them)
        out["decode_other_workloads"] = decode_other_workloads(torch, dev, numbers=(3, 4, 5))
        out["decode_other_workloads"]["note"] = ("each batch's decode launches alone (a few layers in turn, nothing else on "
                                                 "the GPU); 5 is the main workload's own batch outside the iteration")
        # the 8-bit pool (the paper's future-work direction) on workload 2's shape: write and decode over E4M3 codes
        out["fp8_pool"] = fp8_pool_figures(torch, dev)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_seconds, lens=sorted(dlens)[len(dlens) // 2 - 1:len(dlens) // 2 + 1])
    return out


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.workload != 5:
        full = prefill_decode_workload(args, args.workload, args.steps, args.warmup, component=args.component)
        if args.component:
            full = {k: full[k] for k in ("config", "steps", "warmup", "ms_per_step", "components", "overlap",
                                         "kernels_alone", "roofline", "rooflines_other")}
        print(json.dumps(full))
        return
    # A full step of the two prefill-heavy configurations, so that the same line carries the 16k-token prefill, the
    # 64-step split decode and the offload / reload of whole layers.  Each runs in a process of its own BEFORE this
    # process touches the GPU (one process on the card at a time): a component then measures what `--workload N`
    # alone measures, whatever the 200 GiB of host memory of the main workload leave behind in this process.
    parts = {}
    if not args.no_components and args.kv_dtype == "bf16":
        import subprocess
        for number, steps, warmup in ((2, args.component_steps or 5, 2), (3, args.component_steps or 2, 1)):
            print(f"[bench] component: workload {number}, {warmup} warm-up + {steps} timed steps", file=sys.stderr, flush=True)
            cmd = [sys.executable, os.path.abspath(__file__), "--workload", str(number), "--steps", str(steps),
                   "--warmup", str(warmup), "--component", "--no-cpu-baseline", "--no-extras"]
            r = subprocess.run(cmd, stdout=subprocess.PIPE, text=True)
            lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
            if r.returncode != 0 or not lines:
                print(f"bench.py: the workload {number} component failed (exit {r.returncode})", file=sys.stderr)
                sys.exit(r.returncode or 1)
            parts[f"workload{number}"] = json.loads(lines[-1])
    out = mixed_iteration(args)
    out.update(parts)
    print(json.dumps(out))


def prefill_decode_workload(args, number: int, steps: int, warmup: int, component: bool) -> dict:
    """One step = S0-S6 over the workload's batch: per layer allocate + map, write, causal prefill attention, offload of
    the workload's host layers on a side stream; then their reload and the workload's decode steps.  component: the
    figures the default line carries for workloads 3 and 2 (no CPU baseline, no other-workload extras)."""
    import gc
    import torch
    from paper_2410_00428_amd import workloads as wl
    from paper_2410_00428_amd.engine import LayerKVEngine

    class _A:   # this run's view of the arguments
        pass
    run = _A()
    run.__dict__.update(vars(args))
    run.workload, run.steps, run.warmup = number, steps, warmup
    if component:
        run.no_cpu_baseline, run.no_extras = True, True
    args = run
    w = wl.workload(args.workload)
    sh = w.shape
    L, B = sh.num_layers, len(w.prompt_lens)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    eng_kw = {}
    if args.kv_dtype == "fp8":
        import dataclasses
        w = dataclasses.replace(w, shape=dataclasses.replace(w.shape, dtype="fp8"), name=w.name + "-fp8pool")
        sh = w.shape
        eng_kw = dict(k_scale=w.data_scale / 16, v_scale=w.data_scale / 16)
        args.no_cpu_baseline = True   # the timed oracle sample is the bf16 one
    eng = LayerKVEngine(sh, w.pool_blocks, wl.free_list_order(w.number, w.pool_blocks), **eng_kw)
    T = sum(w.prompt_lens)
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.SEED_BASE + w.number)

    def randn(*shape):
        return (torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32) * w.data_scale).to(torch.bfloat16)

    # inputs of every layer resident in HBM before timing (layers get their own tensors so that the
    # per-layer working set is not served from cache)
    n_in = L if T * sh.num_q_heads * sh.head_dim * 2 * 3 * L < 64 * 2**30 else 4
    Qs = [randn(T, sh.num_q_heads, sh.head_dim) for _ in range(n_in)]
    Ks = [randn(T, sh.num_kv_heads, sh.head_dim) for _ in range(n_in)]
    Vs = [randn(T, sh.num_kv_heads, sh.head_dim) for _ in range(n_in)]
    O = torch.empty_like(Qs[0])
    dq = [randn(B, sh.num_q_heads, sh.head_dim) for _ in range(L)]
    dk = [randn(B, sh.num_kv_heads, sh.head_dim) for _ in range(L)]
    dv = [randn(B, sh.num_kv_heads, sh.head_dim) for _ in range(L)]
    dO = torch.empty_like(dq[0])
    off_layers = [] if args.no_offload else list(w.offload_layers)
    layer_bytes = sum(wl.blocks_for(n, sh.block_size) for n in w.prompt_lens) * sh.block_bytes
    pinned = {l: eng.pinned(layer_bytes) for l in off_layers}

    def step(after_layer=None):
        eng.reset()
        eng.begin_prompts(w.prompt_lens)
        eng.prefill_all_layers(Qs, Ks, Vs, O, pinned, after_layer)
        for l in off_layers:
            eng.release_offloaded(l)
        for l in off_layers:
            eng.reload_layer(l)
        for st in range(w.decode_steps):
            eng.decode_all_layers(dq, dk, dv, dO, step=st)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Timed steps: the library's own events around its launches, and events from here only around the side-stream
    # transfers (for their spans).  Events from Python around the main-stream calls as well would put two more
    # packets next to every launch; they are taken in one extra, untimed step afterwards, for comparison.
    eng.timing = "side"
    eng.timers.clear()
    eng.ctx.set_profiling(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    side_timers = dict(eng.timers)
    stats = eng.ctx.get_stats()
    eng.ctx.set_profiling(False)
    eng.timing = True
    eng.timers.clear()
    step()
    ms = eng.elapsed_ms()
    eng.timing = False

    K = args.steps
    def total(name):
        return sum(ms.get(name, [0.0]))
    def avg(name):
        v = ms.get(name, [])
        return sum(v) / len(v) if v else float("nan")

    decode_ctx = [[n + st + 1 for n in w.prompt_lens] for st in range(w.decode_steps)]
    decode_bytes_per_launch = [sum(c) * sh.token_bytes for c in decode_ctx]
    decode_bytes_total = sum(decode_bytes_per_launch) * L * K
    # Kernel time = the library's own HIP events, attached to the kernels of each launch (lkv_set_profiling: the
    # start event takes the kernel's begin, the stop event its end, as a profiler reports it).  Events recorded
    # from Python around the C call (eng.timers) also contain the stream's hand-over before and after a launch and
    # the time the GPU waits for the interpreter between two launches; they are kept for comparison.
    decode_ms_lib = stats["decode_kernel_ns"] * 1e-6
    assert stats["decode_kernel_launches"] == L * K * w.decode_steps
    decode_gbs = decode_bytes_total / (decode_ms_lib * 1e-3) / 1e9
    decode_gbs_py = decode_bytes_total / K / (total("decode_attention") * 1e-3) / 1e9   # one step
    pf_flops = causal_flops(w.prompt_lens, sh.num_q_heads, sh.head_dim)
    assert stats["prefill_kernel_launches"] == L * K
    prefill_ms_lib = stats["prefill_kernel_ns"] * 1e-6 / (L * K)
    prefill_tflops = pf_flops / (prefill_ms_lib * 1e-3) / 1e12
    prefill_tflops_py = pf_flops / (avg("prefill_attention") * 1e-3) / 1e12
    # write_kv is called for the prompts (T tokens) and for every decode step (B tokens); only the former count
    write_gbs = stats["write_kernel_bytes"] / max(stats["write_kernel_ns"], 1)     # library events; includes the
    # few-microsecond launches that append the decode step's tokens (about 5 % of the time, none of the bytes)
    write_gbs_py = 2 * T * sh.token_bytes / (avg("write_kv") * 1e-3) / 1e9
    pack_gbs = stats["pack_kernel_bytes"] / max(stats["pack_kernel_ns"], 1)      # bytes/ns = GB/s
    unpack_gbs = stats["unpack_kernel_bytes"] / max(stats["unpack_kernel_ns"], 1)

    def span_ms(name):  # first start -> last end of a side-stream activity, per step
        v = side_timers.get(name, [])
        per = len(v) // K if K else 0
        if not per:
            return float("nan")
        return sum(v[i * per][0].elapsed_time(v[i * per + per - 1][1]) for i in range(K)) / K
    off_ms, rel_ms = span_ms("offload"), span_ms("reload")

    def steady_gbs(name):
        """Host-link rate of a side-stream transfer phase once it is running: the bytes of all layers but the first over
        the time from the end of the first layer's transfer to the end of the last one's.  (The span from the first
        call's start also holds what the first transfer waits for: in workload 2's step the offload stream is free
        from the start of the phase, so its first event is 7 ms older than the first copy.)"""
        v = side_timers.get(name, [])
        per = len(v) // K if K else 0
        if per < 2:
            return None
        t = sum(v[i * per][1].elapsed_time(v[i * per + per - 1][1]) for i in range(K)) / K
        return layer_bytes * (per - 1) / (t * 1e-3) / 1e9
    # prefill launches up to the first offloaded layer vs the later ones (a copy is then running next to them); the
    # first group also holds the clock transient after the idle gap at the start of the phase
    pf = ms.get("prefill_attention", [])
    first_off = min(off_layers) if off_layers else L
    pf_quiet = [t for i, t in enumerate(pf) if i % L <= first_off]
    pf_overlap = [t for i, t in enumerate(pf) if i % L > first_off]
    off_gbs = steady_gbs("offload") if off_layers else None
    rel_gbs = steady_gbs("reload") if off_layers else None

    # ---- outside the timed steps: the host link's own peak, and how much of the offload hides behind prefill
    def ev():
        return torch.cuda.Event(enable_timing=True)
    link = pinned_copy_peak(torch, dev)

    def prefill_phase(offload):
        """offload: False, True (the workload's layers) or an explicit {layer: pinned buffer}."""
        eng.reset()
        eng.begin_prompts(w.prompt_lens)
        a, b, d = ev(), ev(), ev()
        a.record(eng.main)
        eng.prefill_all_layers(Qs, Ks, Vs, O, offload if isinstance(offload, dict) else (pinned if offload else {}))
        b.record(eng.main)
        d.record(eng.d2h)
        torch.cuda.synchronize()
        return a.elapsed_time(b), max(a.elapsed_time(b), a.elapsed_time(d))
    overlap = None
    iso = {}
    write_gbs_prompts = None
    if off_layers:
        prefill_phase(False)
        t_compute, _ = prefill_phase(False)
        eng.ctx.set_profiling(True)
        s0 = eng.ctx.get_stats()
        a, b = ev(), ev()
        a.record(eng.d2h)
        for l in off_layers:
            eng.offload_layer(l, pinned[l])
        b.record(eng.d2h)
        torch.cuda.synchronize()
        t_link = a.elapsed_time(b)
        s1 = eng.ctx.get_stats()
        iso["pack_kernel_GBps"] = (s1["pack_kernel_bytes"] - s0["pack_kernel_bytes"]) / max(
            s1["pack_kernel_ns"] - s0["pack_kernel_ns"], 1)
        # reload alone: nothing else on the GPU
        for l in off_layers:
            eng.release_offloaded(l)
        a, b = ev(), ev()
        a.record(eng.h2d)
        for l in off_layers:
            eng.reload_layer(l)
        b.record(eng.h2d)
        torch.cuda.synchronize()
        t_reload = a.elapsed_time(b)
        s2 = eng.ctx.get_stats()
        eng.ctx.set_profiling(False)
        iso["unpack_kernel_GBps"] = (s2["unpack_kernel_bytes"] - s1["unpack_kernel_bytes"]) / max(
            s2["unpack_kernel_ns"] - s1["unpack_kernel_ns"], 1)
        iso["offload_GBps"] = layer_bytes * len(off_layers) / (t_link * 1e-3) / 1e9
        iso["reload_GBps"] = layer_bytes * len(off_layers) / (t_reload * 1e-3) / 1e9
        # the same layers through the pageable tier: ordinary host memory behind the library's small pinned ring
        pageable = np.ones(layer_bytes * len(off_layers) if not component else 0, dtype=np.uint8)   # touched before timing
        views = {l: pageable[i * layer_bytes:(i + 1) * layer_bytes] for i, l in enumerate(off_layers)}
        t_page = {}
        for rep in range(0 if component else 2):                            # first pass builds the ring
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for l in off_layers:
                eng.offload_layer_pageable(l, views[l])
            eng.ctx.host_tier_synchronize()
            t_page["offload"] = time.perf_counter() - t0
            same = all(bytes(views[l][:4096]) == bytes(pinned[l][:4096].numpy()) and
                       bytes(views[l][-4096:]) == bytes(pinned[l][layer_bytes - 4096:layer_bytes].numpy())
                       for l in off_layers)
            for l in off_layers:
                eng.release_offloaded(l)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for l in off_layers:
                eng.reload_layer(l)
            torch.cuda.synchronize()
            t_page["reload"] = time.perf_counter() - t0
        s3 = eng.ctx.get_stats()
        for l in off_layers:
            eng.host_images[l] = pinned[l]
        if not component:
          iso["pageable_tier"] = {
              "offload_GBps": round(layer_bytes * len(off_layers) / t_page["offload"] / 1e9, 2),
              "reload_GBps": round(layer_bytes * len(off_layers) / t_page["reload"] / 1e9, 2),
              "pinned_ring_MiB": 128, "host_image_MiB": pageable.nbytes >> 20,
              "memcpy_GBps_per_thread": round(s3["tier_copy_bytes"] / max(s3["tier_copy_ns"], 1), 1),
              "image_ends_equal_pinned_path": bool(same),
              "note": "lkv_offload_layer_pageable / lkv_reload_layer_pageable: wall time until the image is complete "
                      "in ordinary host memory (4 CPU threads drain 4 pinned units of 32 MiB), resp. until the blocks "
                      "are back in the pool"}
        del pageable, views
        _, t_both = prefill_phase(True)
        # the same phase once more with the library's events on: the prompt writes by themselves (the step's
        # write statistics also hold the few-microsecond launches that append each decode step's tokens)
        eng.ctx.set_profiling(True)
        p0 = eng.ctx.get_stats()
        prefill_phase(True)
        p1 = eng.ctx.get_stats()
        eng.ctx.set_profiling(False)
        write_gbs_prompts = (p1["write_kernel_bytes"] - p0["write_kernel_bytes"]) / max(
            p1["write_kernel_ns"] - p0["write_kernel_ns"], 1)
        # only the compute issued after the first offload can hide anything
        t_hideable = t_compute * (L - 1 - first_off) / L
        overlap = {"prefill_compute_ms": round(t_compute, 3), "offload_link_ms": round(t_link, 3),
                   "both_ms": round(t_both, 3),
                   "hidden_frac": round(max(0.0, 1 - (t_both - t_compute) / t_link), 4),
                   "bound": round(min(1.0, t_hideable / t_link), 4),
                   "hidden_over_bound": round(max(0.0, 1 - (t_both - t_compute) / t_link) / max(min(1.0, t_hideable / t_link), 1e-9), 4),
                   "note": "hidden = 1 - (wall(prefill with offload) - wall(prefill alone)) / wall(offload alone); bound = "
                           "compute issued after the first offload starts / link time: attention-only compute cannot "
                           "hide a PCIe transfer of the same layers"}
        # The paper's own answer to that (Section 3.2.1): retain x layers, x the smallest number whose offload
        # time does not exceed the prefill time.  Both models are fitted to THIS run: alpha from the measured
        # prefill phase (attention only: no weights on this path, n_param = 0), beta from the measured link time.
        from paper_2410_00428_amd import binding as lkv_b
        n_tok = sum(w.prompt_lens)
        cm = lkv_b.CostModel(alpha=1.0, n_param=0.0, n_hidden=float(L * sh.num_q_heads * sh.head_dim),
                             device_flops=MFMA_BF16_PEAK_TFLOPS * 1e12, beta=1.0, num_layers=L, head_dim=sh.head_dim,
                             num_heads=sh.num_kv_heads, bytes_per_elem=2.0, link_bytes_per_s=link["d2h"] * 1e9)
        # the batch is B equal prompts: per-request times are the phase times divided by B
        s_req = w.prompt_lens[0]
        cm.alpha = (t_compute * 1e-3 / B) / lkv_b.prefill_time(cm, s_req)
        cm.beta = (t_link * 1e-3 / B) / lkv_b.offload_time(cm, s_req, L - len(off_layers))
        x_plan, mask = lkv_b.plan_offload(cm, s_req)
        planned = [l for l in range(L) if not mask[l]]
        plan = {"alpha": round(cm.alpha, 3), "beta": round(cm.beta, 3), "retain_x": x_plan, "offloaded_layers": planned,
                "retain_x_at_16k_tokens": lkv_b.plan_offload(cm, 16384)[0]}
        if planned:
            plan_bufs = {l: pinned[off_layers[i % len(off_layers)]] for i, l in enumerate(planned)}
            eng.reset()
            eng.begin_prompts(w.prompt_lens)
            eng.prefill_all_layers(Qs, Ks, Vs, O, {})
            torch.cuda.synchronize()
            a, b = ev(), ev()
            a.record(eng.d2h)
            for l in planned:
                eng.offload_layer(l, plan_bufs[l])
            b.record(eng.d2h)
            torch.cuda.synchronize()
            t_link_plan = a.elapsed_time(b)          # the planned layers' pack + copy with nothing else running
            prefill_phase(plan_bufs)                 # first run of a new pattern: not timed
            _, t_both_plan = prefill_phase(plan_bufs)
            plan.update({"offload_link_ms": round(t_link_plan, 3), "both_ms": round(t_both_plan, 3),
                         "hidden_frac": round(max(0.0, min(1.0, 1 - (t_both_plan - t_compute) / t_link_plan)), 4)})
        overlap["planned_by_lkv_plan_offload"] = plan

    # kernels alone, launched back to back (no other stream active, no events between launches)
    def alone(fn, launches, reps=3):
        fn()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record(eng.main)
        for _ in range(reps):
            fn()
        b.record(eng.main)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / (reps * launches)
    eng.reset()
    eng.begin_prompts(w.prompt_lens)
    slots_all = torch.from_numpy(np.stack([eng.map_prefill_layer(l) for l in range(L)])).to(dev)
    c = eng.ctx
    slot_rows = [slots_all[l] for l in range(L)]          # views made outside the timed loops
    t_write = alone(lambda: [c.write_kv(l, Ks[l % n_in], Vs[l % n_in], slot_rows[l], T, eng.main) for l in range(L)], L)
    t_prefill = alone(lambda: [c.prefill_attention(l, Qs[l % n_in], Ks[l % n_in], Vs[l % n_in], O, eng.cu_dev, B,
                                                   max(w.prompt_lens), T, True, eng.main) for l in range(L)], L)
    maps = [eng.map_decode_layer(l, 0) for l in range(L)]
    bt_all = torch.from_numpy(np.stack([m[1] for m in maps])).to(dev)
    cl_dev = torch.from_numpy(np.asarray([n + 1 for n in w.prompt_lens], dtype=np.int32)).to(dev)
    bt_rows, bt_w = [bt_all[l] for l in range(L)], bt_all.shape[2]
    t_decode = alone(lambda: [c.paged_decode_attention(l, dq[l], dO, bt_rows[l], bt_w, cl_dev, B, eng.main)
                              for l in range(L)], L, reps=5)
    iso["write_kv_GBps_back_to_back_from_python"] = 2 * T * sh.token_bytes / (t_write * 1e-3) / 1e9
    # an 80 us kernel launched from Python is partly launch-bound; the kernel itself, by the library's events:
    c.set_profiling(True)
    w0 = c.get_stats()
    for l in range(L):
        c.write_kv(l, Ks[l % n_in], Vs[l % n_in], slot_rows[l], T, eng.main)
    w1 = c.get_stats()
    c.set_profiling(False)
    iso["write_kv_GBps"] = (w1["write_kernel_bytes"] - w0["write_kernel_bytes"]) / max(
        w1["write_kernel_ns"] - w0["write_kernel_ns"], 1)
    iso["prefill_attn_TFLOPs"] = pf_flops / (t_prefill * 1e-3) / 1e12
    iso["decode_paged_attn_GBps"] = decode_bytes_per_launch[0] / (t_decode * 1e-3) / 1e9
    iso = {k: (round(v, 2) if isinstance(v, float) else v) for k, v in iso.items()}
    traffic = measured_traffic("prefill_bf16_d128_kernel", args.workload) if args.kv_dtype == "bf16" else None
    torch.cuda.synchronize()
    others = None if args.no_extras else decode_other_workloads(torch, dev)
    fp8_fig = None if args.no_extras else fp8_pool_figures(torch, dev)

    out = {
        "metric": METRIC, "value": round(decode_gbs, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": round(wall * 1e3 / K, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {w.name} (L={L}, Hq={sh.num_q_heads}, Hkv={sh.num_kv_heads}, "
                               f"d={sh.head_dim}, block 16, {B} prompts x {w.prompt_lens[0]} tokens, "
                               f"{len(off_layers)} layers offloaded+reloaded, {w.decode_steps} decode step(s))",
                   "value_is": "decode paged attention: context KV bytes (K and V once per kv head) / HIP-event time "
                               "of the decode launches (events attached by the library to each launch's kernels: begin "
                               "of the first, end of the last), measured inside the full step"},
        "components": {
            "decode_paged_attn_GBps": round(decode_gbs, 2),
            "decode_frac_of_hbm_peak": round(decode_gbs / HBM_PEAK_GBS, 4),
            "decode_us_per_layer": round(decode_ms_lib * 1e3 / (L * K * w.decode_steps), 2),
            "decode_paged_attn_GBps_events_from_python": round(decode_gbs_py, 2),
            "prefill_attn_TFLOPs": round(prefill_tflops, 2),
            "prefill_frac_of_bf16_mfma_peak": round(prefill_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
            "prefill_ms_per_layer": round(prefill_ms_lib, 4),
            "prefill_attn_TFLOPs_events_from_python": round(prefill_tflops_py, 2),
            "prefill_ms_per_layer_up_to_first_offload": round(sum(pf_quiet) / max(len(pf_quiet), 1), 4),
            "prefill_ms_per_layer_after_first_offload": round(sum(pf_overlap) / max(len(pf_overlap), 1), 4),
            "write_kv_GBps": round(write_gbs, 2),
            "write_kv_GBps_prompt_writes": round(write_gbs_prompts, 2) if write_gbs_prompts else None,
            "write_kv_GBps_events_from_python": round(write_gbs_py, 2),
            "write_kv_us_per_layer_events_from_python": round(avg("write_kv") * 1e3, 2),
            "pack_kernel_GBps": round(pack_gbs, 2), "unpack_kernel_GBps": round(unpack_gbs, 2),
            "offload_GBps": None if off_gbs is None else round(off_gbs, 2),
            "reload_GBps": None if rel_gbs is None else round(rel_gbs, 2),
            "offload_ms_first_call_to_last_end": None if off_gbs is None else round(off_ms, 2),
            "reload_ms_first_call_to_last_end": None if rel_gbs is None else round(rel_ms, 2),
            "pinned_copy_peak_GBps": {k: round(v, 2) for k, v in link.items()},
            "offload_frac_of_link_peak": None if off_gbs is None else round(off_gbs / link["d2h"], 4),
            "reload_frac_of_link_peak": None if rel_gbs is None else round(rel_gbs / link["h2d"], 4),
        },
        "overlap": overlap,
        "kernels_alone": dict(iso, note="each kernel launched back to back with nothing else on the GPU; the "
                                        "components above are measured inside the full step, where streams overlap"),
        "roofline": {"kernel": "prefill_bf16_d128_kernel (lkv_prefill_attention)", "bound": "mfma",
                     "achieved": round(prefill_tflops, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(prefill_tflops / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic,
                     "launch_ms": round(prefill_ms_lib, 4), "flops_per_launch": pf_flops},
        "rooflines_other": {
            "decode": {"bound": "hbm", "achieved": round(decode_gbs, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": round(decode_gbs / HBM_PEAK_GBS, 4)},
            "write_kv": {"bound": "hbm", "achieved": round(write_gbs_prompts or write_gbs, 2), "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": round((write_gbs_prompts or write_gbs) / HBM_PEAK_GBS, 4),
                         "launches": "the prompt writes of the prefill phase, offload running" if write_gbs_prompts
                                     else "all write launches of the step"},
            "pack": {"bound": "hbm", "achieved": round(pack_gbs, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(pack_gbs / HBM_PEAK_GBS, 4)},
            "unpack": {"bound": "hbm", "achieved": round(unpack_gbs, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": round(unpack_gbs / HBM_PEAK_GBS, 4)},
        },
        "decode_other_workloads": others,
        "fp8_pool": fp8_fig,
    }
    eng.close()
    del eng, Qs, Ks, Vs, O, dq, dk, dv, dO, pinned, slots_all, slot_rows, bt_all, bt_rows
    gc.collect()
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_seconds)
    return out


if __name__ == "__main__":
    main()
