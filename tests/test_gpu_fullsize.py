"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py times (through
``LayerKVEngine``), on outputs the oracle can compute one by one: sampled causal rows, whole decode
steps, byte-exact pools and offload images.  Workloads 2-5; where a workload is cut down for the
CPU side's sake the deviation is stated in the test."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import layerkv_oracle as orc  # noqa: E402
from paper_2410_00428_amd import binding as lkv  # noqa: E402
from paper_2410_00428_amd import workloads as wl  # noqa: E402
from paper_2410_00428_amd.engine import LayerKVEngine  # noqa: E402
from tests import gpu_harness as H  # noqa: E402

pytestmark = pytest.mark.gpu
THREADS = 16


def say(msg: str) -> None:
    """Progress of the minute-long tests (seen with pytest -s; a silent GPU run is taken for a hung one)."""
    print(f"[fullsize] {msg}", flush=True)


def sampled_prefill_check(cfg, layer, Q, K, V, O_dev, lens, shape, scale, triples, rows_per=64):
    """>= 64 rows (always 0, 15, 16, n-1) for each of the given (sequence, head) pairs."""
    cu = wl.cu_seqlens(lens)
    rng = wl.rng_for(cfg, "lengths", 1000 + layer)
    tok, head = [], []
    for s, h in triples:
        rows = wl.sample_rows(rng, lens[s], rows_per)
        tok += [int(cu[s] + r) for r in rows]
        head += [h] * len(rows)
    ref = orc.prefill_attention_rows(Q, K, V, cu, shape.dtype, tok, head, threads=THREADS)
    got = H.to_host(O_dev[torch.tensor(tok, device=H.DEV), torch.tensor(head, device=H.DEV)], shape.dtype)
    H.check_attention(got, ref, shape.dtype, scale, f"sampled prefill rows, layer {layer}")


def pool_blocks_equal(pool_dev, o, ids, what):
    ids = np.asarray(ids)
    blocks = pool_dev.view(o.num_pool_blocks, -1)[torch.from_numpy(ids.astype(np.int64)).to(H.DEV)].cpu().numpy()
    assert blocks.tobytes() == o.pool[ids].tobytes(), f"{what}: pool blocks differ"


def upload_blocks(pool_dev, o, ids):
    ids = np.asarray(ids)
    src = torch.from_numpy(o.pool[ids].reshape(len(ids), -1).view(np.uint8))
    pool_dev.view(o.num_pool_blocks, -1)[torch.from_numpy(ids.astype(np.int64)).to(H.DEV)] = src.to(H.DEV)


def fill_blocks_random(o, ids, rng, scale):
    """Seeded values for whole blocks, written straight into the oracle's pool (the write path has its own
    tests); a 4 Mi-element draw is tiled so that GiB-sized pools do not cost minutes of CPU time."""
    chunk = wl.normal_tensor(rng, (1 << 22,), scale, o.dtype)
    per = o.pool[0].size
    reps = -(-len(ids) * per // chunk.size)
    flat = np.tile(chunk, reps)[: len(ids) * per].reshape((len(ids),) + o.pool.shape[1:])
    o.pool[np.asarray(ids)] = flat


# ----------------------------------------------------------------------------- workload 2
def test_workload2_full_size_two_layers_through_the_engine():
    """8 x 2048 prompts, LLaMA-2-7B shape, full pool: layers 3 (kept) and 17 (offloaded, freed, reloaded into
    other blocks) go through exactly the calls bench.py issues; one decode step on both."""
    w = wl.workload(2)
    sh, lens = w.shape, list(w.prompt_lens)
    order = wl.free_list_order(2, w.pool_blocks)
    pool = torch.zeros(w.pool_blocks * sh.block_bytes, dtype=torch.uint8, device=H.DEV)
    eng = LayerKVEngine(sh, w.pool_blocks, order, pool=pool)
    o = orc.LayerKVOracle(sh.num_layers, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.block_size,
                          w.pool_blocks, sh.dtype)
    o.pool_reset(order)
    eng.begin_prompts(lens)
    T = sum(lens)
    layer_bytes = sum(wl.blocks_for(n, 16) for n in lens) * sh.block_bytes
    pinned = eng.pinned(layer_bytes)
    for layer in (3, 17):
        Q, K, V = wl.qkv(2, layer, T, sh, w.data_scale)
        Qd, Kd, Vd = H.to_dev(Q), H.to_dev(K), H.to_dev(V)
        Od = H.empty_like_storage(Q.shape, sh.dtype)
        eng.prefill_layer(layer, Qd, Kd, Vd, Od, offload_to=pinned if layer == 17 else None)
        for s, n in enumerate(lens):
            o.alloc_layer_blocks(s, layer, n)
            assert eng.ctx.get_block_table(s, layer).tolist() == o.block_table(s, layer)
        slots = np.concatenate([o.slot_mapping(s, layer, 0, n) for s, n in enumerate(lens)])
        o.write_kv(K, V, slots)
        torch.cuda.synchronize()
        sampled_prefill_check(2, layer, Q, K, V, Od, lens, sh, w.data_scale,
                              [(0, 0), (1, 5), (2, 31), (3, 16), (4, 7), (5, 8), (6, 23), (7, 30)])
        ids = sum((o.block_table(s, layer) for s in range(len(lens))), [])
        pool_blocks_equal(pool, o, ids, f"after write, layer {layer}")
    # offload image of layer 17, then free + reload elsewhere
    eng.ctx.event_synchronize(17, lkv.LKV_EV_OFFLOADED)
    old_ids = sum((o.block_table(s, 17) for s in range(len(lens))), [])
    image = o.pack_layer_blocks(old_ids).copy()
    assert pinned.numpy().tobytes() == image.tobytes(), "offload image differs"
    eng.release_offloaded(17)
    for s in range(len(lens)):
        o.free_layer_blocks(s, 17, to_host=True)
    eng.ctx.alloc_layer_blocks(777, 0, 16 * 37)      # someone else takes 37 blocks in between
    o.alloc_layer_blocks(777, 0, 16 * 37)
    eng.reload_layer(17)
    for s, n in enumerate(lens):
        o.alloc_layer_blocks(s, 17, n)
    new_ids = sum((o.block_table(s, 17) for s in range(len(lens))), [])
    assert new_ids != old_ids
    o.unpack_layer_blocks(new_ids, image)
    for layer in (3, 17):
        q, k, v = wl.decode_qkv(2, layer, 0, len(lens), sh, w.data_scale)
        Od = H.empty_like_storage(q.shape, sh.dtype)
        eng.decode_layer(layer, H.to_dev(q), H.to_dev(k), H.to_dev(v), Od)
        slots = []
        for s, n in enumerate(lens):
            o.alloc_layer_blocks(s, layer, n + 1)
            assert eng.ctx.get_block_table(s, layer).tolist() == o.block_table(s, layer)
            slots.append(o.slot_mapping(s, layer, n, 1))
        o.write_kv(k, v, np.concatenate(slots))
        bt = o.padded_block_table(range(len(lens)), layer)
        ref = o.paged_decode_attention(q, bt, [n + 1 for n in lens], threads=THREADS)
        torch.cuda.synchronize()
        H.check_attention(H.to_host(Od, sh.dtype), ref, sh.dtype, w.data_scale, f"decode layer {layer}")
        ids = sum((o.block_table(s, layer) for s in range(len(lens))), [])
        pool_blocks_equal(pool, o, ids, f"after decode append, layer {layer}")
    eng.close()


# ----------------------------------------------------------------------------- workload 3
def test_workload3_long_context_prefill_rows_and_split_decode():
    """16384-token prompts: sampled causal rows of one full-length prompt at the 7B head count, and the
    4 x 16385 split-K decode of one layer, every output row."""
    w = wl.workload(3)
    sh = w.shape
    # prefill: one 16384-token prompt (the workload has four; one gives the same launch shape per sequence)
    n = 16384
    Q, K, V = wl.qkv(3, 0, n, sh, w.data_scale)
    c = lkv.LKV(1, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, 16, 64, "bf16")
    Od = H.empty_like_storage(Q.shape, "bf16")
    c.prefill_attention(0, H.to_dev(Q), H.to_dev(K), H.to_dev(V), Od, H.to_dev(wl.cu_seqlens([n])), 1, n, n, True)
    torch.cuda.synchronize()
    sampled_prefill_check(3, 0, Q, K, V, Od, [n], sh, w.data_scale, [(0, h) for h in (0, 3, 9, 14, 17, 22, 28, 31)])
    c.destroy()
    # decode: 4 sequences, context 16385, one layer's worth of pool
    lens = [16385] * 4
    nblk = sum(wl.blocks_for(m, 16) for m in lens) + 64
    one = wl.KVShape(1, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, 16, "bf16")
    order = wl.free_list_order(3, nblk)
    cd, o, pool = H.make_pair(one, nblk, order)
    for s, m in enumerate(lens):
        cd.alloc_layer_blocks(s, 0, m)
        o.alloc_layer_blocks(s, 0, m)
    ids = sum((o.block_table(s, 0) for s in range(4)), [])
    fill_blocks_random(o, ids, wl.rng_for(3, "k", 99), w.data_scale)
    upload_blocks(pool, o, ids)
    q, _, _ = wl.decode_qkv(3, 0, 0, 4, sh, w.data_scale, q_gain=8.0)
    bt = cd.padded_block_table(range(4), 0)
    assert np.array_equal(bt, o.padded_block_table(range(4), 0))
    Od = H.empty_like_storage(q.shape, "bf16")
    cd.paged_decode_attention(0, H.to_dev(q), Od, H.to_dev(bt), bt.shape[1], H.to_dev(np.asarray(lens, np.int32)), 4)
    ref = o.paged_decode_attention(q, bt, lens, threads=THREADS)
    torch.cuda.synchronize()
    H.check_attention(H.to_host(Od, "bf16"), ref, "bf16", w.data_scale, "workload 3 decode")
    cd.destroy()


# ----------------------------------------------------------------------------- workload 4
def test_workload4_gqa_decode_with_fragmented_per_layer_tables():
    """LLaMA-2-70B KV shape (64 q heads on 8 kv heads), 16 lognormal contexts, tables built by the seeded
    fragmenting schedule with a different permutation per layer; two of the 80 layers, every output row."""
    w = wl.workload(4)
    sh, lens = w.shape, list(w.decode_lens)
    L = 2
    per_layer = sum(wl.blocks_for(n, 16) for n in lens)
    nblk = int(per_layer * L * 1.25) + 1024
    two = wl.KVShape(L, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, 16, "bf16")
    order = wl.free_list_order(4, nblk)
    c, o, pool = H.make_pair(two, nblk, order)
    for layer in range(L):
        for op in wl.fragmenting_schedule(4, layer, lens, 16):
            if op.op == "alloc":
                c.alloc_layer_blocks(op.seq, op.layer, op.tokens)
                o.alloc_layer_blocks(op.seq, op.layer, op.tokens)
            else:
                c.free_layer_blocks(op.seq, op.layer, False)
                o.free_layer_blocks(op.seq, op.layer)
    jumps = total = 0
    for layer in range(L):
        ids = sum((o.block_table(s, layer) for s in range(len(lens))), [])
        fill_blocks_random(o, ids, wl.rng_for(4, "k", 50 + layer), w.data_scale)
        upload_blocks(pool, o, ids)
        bt = c.padded_block_table(range(len(lens)), layer)
        assert np.array_equal(bt, o.padded_block_table(range(len(lens)), layer))
        for s in range(len(lens)):
            t = np.asarray(o.block_table(s, layer))
            jumps += int((np.diff(t) != 1).sum())
            total += len(t) - 1
        q, _, _ = wl.decode_qkv(4, layer, 0, len(lens), sh, w.data_scale, q_gain=8.0)
        Od = H.empty_like_storage(q.shape, "bf16")
        c.paged_decode_attention(layer, H.to_dev(q), Od, H.to_dev(bt), bt.shape[1],
                                 H.to_dev(np.asarray(lens, np.int32)), len(lens))
        ref = o.paged_decode_attention(q, bt, lens, threads=THREADS)
        torch.cuda.synchronize()
        H.check_attention(H.to_host(Od, "bf16"), ref, "bf16", w.data_scale, f"workload 4 decode layer {layer}")
    assert jumps / total >= 0.5, "tables are not fragmented"
    assert o.block_table(0, 0) != o.block_table(0, 1)
    c.destroy()


# ----------------------------------------------------------------------------- workload 5
def test_workload5_mixed_batch_reload_on_side_stream_while_decoding():
    """Mixed serving iteration at the 7B shape, cut down for the CPU side: the first 16 of the 64 decode
    sequences (lengths uniform in [128, 16384]) and the 2 new 8192-token prompts, three layers of which two
    start host-resident.  Per layer: reload on the side stream (if host-resident) -> paged decode -> write +
    prefill of the new prompts -> offload of their blocks on the other side stream."""
    w = wl.workload(5)
    sh = w.shape
    dlens = list(w.decode_lens[:16])
    plens = list(w.prompt_lens)
    L = 3
    three = wl.KVShape(L, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, 16, "bf16")
    per_layer = sum(wl.blocks_for(n + 1, 16) for n in dlens) + sum(wl.blocks_for(n, 16) for n in plens)
    nblk = per_layer * L + 256
    order = wl.free_list_order(5, nblk)
    c, o, pool = H.make_pair(three, nblk, order)
    d2h, h2d = torch.cuda.Stream(), torch.cuda.Stream()
    B = len(dlens)
    host_resident = (0, 2)
    images = {}
    # initial state: decode sequences' KV exists; layers 0 and 2 live in pinned host memory
    for layer in range(L):
        for s, n in enumerate(dlens):
            c.alloc_layer_blocks(s, layer, n)
            o.alloc_layer_blocks(s, layer, n)
        ids = sum((o.block_table(s, layer) for s in range(B)), [])
        fill_blocks_random(o, ids, wl.rng_for(5, "k", 70 + layer), w.data_scale)
        if layer in host_resident:
            img = o.pack_layer_blocks(ids).copy()
            buf = H.pinned_bytes(img.nbytes)
            buf.numpy()[:] = img
            images[layer] = (buf, img)
            for s in range(B):
                c.free_layer_blocks(s, layer, True)
                o.free_layer_blocks(s, layer, to_host=True)
        else:
            upload_blocks(pool, o, ids)
    T = sum(plens)
    cu = wl.cu_seqlens(plens)
    cu_dev = H.to_dev(cu)
    new_images = {}
    for layer in range(L):
        if layer in host_resident:
            for s, n in enumerate(dlens):
                c.alloc_layer_blocks(s, layer, n)
                o.alloc_layer_blocks(s, layer, n)
            ids = sum((o.block_table(s, layer) for s in range(B)), [])
            assert ids == sum((c.get_block_table(s, layer).tolist() for s in range(B)), [])
            c.unpack_layer_blocks(layer, ids, images[layer][0], h2d)     # decode below waits for it
            o.unpack_layer_blocks(ids, images[layer][1])
        q, _, _ = wl.decode_qkv(5, layer, 0, B, sh, w.data_scale, q_gain=0.25)
        bt = c.padded_block_table(range(B), layer)
        Od = H.empty_like_storage(q.shape, "bf16")
        c.paged_decode_attention(layer, H.to_dev(q), Od, H.to_dev(bt), bt.shape[1],
                                 H.to_dev(np.asarray(dlens, np.int32)), B)
        # the two new prompts of this iteration
        Q, K, V = wl.qkv(5, layer, T, sh, w.data_scale, q_gain=0.25)
        slots = []
        for i, n in enumerate(plens):
            c.alloc_layer_blocks(100 + i, layer, n)
            o.alloc_layer_blocks(100 + i, layer, n)
            slots.append(c.build_slot_mapping(100 + i, layer, 0, n))
            assert np.array_equal(slots[-1], o.slot_mapping(100 + i, layer, 0, n))
        slots = np.concatenate(slots)
        Qd, Kd, Vd = H.to_dev(Q), H.to_dev(K), H.to_dev(V)
        Op = H.empty_like_storage(Q.shape, "bf16")
        c.write_kv(layer, Kd, Vd, H.to_dev(slots), T)
        c.prefill_attention(layer, Qd, Kd, Vd, Op, cu_dev, len(plens), max(plens), T, True)
        o.write_kv(K, V, slots)
        pids = sum((o.block_table(100 + i, layer) for i in range(len(plens))), [])
        buf = H.pinned_bytes(len(pids) * sh.block_bytes)
        c.pack_layer_blocks(layer, pids, buf, d2h)                       # waits for the write on its own
        new_images[layer] = (buf, o.pack_layer_blocks(pids).copy())
        ref = o.paged_decode_attention(q, bt, dlens, threads=THREADS)
        torch.cuda.synchronize()
        H.check_attention(H.to_host(Od, "bf16"), ref, "bf16", w.data_scale, f"workload 5 decode layer {layer}")
        sampled_prefill_check(5, layer, Q, K, V, Op, plens, sh, w.data_scale, [(0, 0), (0, 13), (1, 31), (1, 20)])
    for layer, (buf, ref) in new_images.items():
        c.event_synchronize(layer, lkv.LKV_EV_OFFLOADED)
        assert buf.numpy()[:ref.nbytes].tobytes() == ref.tobytes(), f"offload image of the new prompts, layer {layer}"
    c.destroy()


# ----------------------------------------------------------------------------- mixed-length prefill batch
def test_mixed_length_prefill_batch_at_the_7b_head_count_sampled_rows():
    """The paper's traffic mixes prompt lengths (Section 5.1); a batch of one long prompt among short ones is what
    the slot grid of the d=128 kernel is for (work slots from the total token count, sequences longest first, kv
    heads dealt to the XCDs).  Sampled causal rows of every sequence, including every row of the shortest."""
    sh = wl.SHAPE_7B
    lens = [257, 8192, 64, 1300, 1, 511, 3000, 128, 129, 700]
    T = sum(lens)
    Q, K, V = wl.qkv(5, 3, T, sh, 128 ** -0.5)
    c = lkv.LKV(1, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, 16, 64, "bf16")
    Od = H.empty_like_storage(Q.shape, "bf16")
    Od.fill_(0x7FC0)   # every row must be overwritten
    c.prefill_attention(0, H.to_dev(Q), H.to_dev(K), H.to_dev(V), Od, H.to_dev(wl.cu_seqlens(lens)), len(lens),
                        max(lens), T, True)
    torch.cuda.synchronize()
    got = H.to_host(Od, "bf16")
    assert not np.isnan(got).any(), "a row of O was not written"
    pairs = [(s, h) for s in range(len(lens)) for h in ((3 * s) % 32, 31 - s)]
    sampled_prefill_check(5, 3, Q, K, V, Od, lens, sh, 128 ** -0.5, pairs, rows_per=24)
    c.destroy()


# ----------------------------------------------------------------------------- workload 5 through the ring
def test_workload5_mixed_iteration_through_the_ring_at_the_7b_shape():
    """The iteration ``bench.py --workload 5`` times, at the 7B shape with all 32 layers, 24 of them in ordinary host
    memory behind a ring of three sets of blocks, the two 8192-token prompts prefilled and offloaded alongside - cut
    to the first 8 of the 64 decoding sequences (contexts 3997..13049) for the CPU side's sake.  Checked against the
    oracle on what it can compute one by one: decode rows of the shortest and the longest sequence in a retained and
    two reloaded layers, sampled causal rows of the new prompts, the new prompts' offload image and a decoding
    sequence's stretch of a layer image."""
    from paper_2410_00428_amd.serving import MixedIteration
    from tests.test_gpu_serving import same_tokens
    w = wl.workload(5)
    sh, bs = w.shape, w.shape.block_size
    L = sh.num_layers
    dlens, plens, host = list(w.decode_lens[:8]), list(w.prompt_lens), list(w.offload_layers)
    B, Td, T = len(dlens), sum(dlens), sum(plens)
    dblk = sum(wl.blocks_for(n, bs) for n in dlens)
    pblk = sum(wl.blocks_for(n, bs) for n in plens)
    nblk = (L - len(host) + 3) * dblk + L * pblk + 64
    it = MixedIteration(sh, dlens, plens, host, nblk, ring_layers=3, free_order=wl.free_list_order(5, nblk, index=3),
                        tier_units=4, tier_threads=4)
    scale = w.data_scale
    # one pair of cached tensors for all layers, the roles alternating with the layer's parity; one set of prompts
    A = wl.normal_tensor(wl.rng_for(5, "k", 900), (Td, sh.num_kv_heads, sh.head_dim), scale, "bf16")
    Bt = wl.normal_tensor(wl.rng_for(5, "v", 900), (Td, sh.num_kv_heads, sh.head_dim), scale, "bf16")
    kv_of = lambda l: (A, Bt) if l % 2 == 0 else (Bt, A)
    Ad, Bd = H.to_dev(A), H.to_dev(Bt)
    q_host = [wl.decode_qkv(5, l, 0, B, sh, scale, q_gain=0.25)[0] for l in range(L)]
    q_dev = [H.to_dev(q) for q in q_host]
    Q, K, V = wl.qkv(5, 901, T, sh, scale, q_gain=0.25)
    Qd, Kd, Vd = H.to_dev(Q), H.to_dev(K), H.to_dev(V)
    it.build_cached_state(lambda l: (Ad, Bd) if l % 2 == 0 else (Bd, Ad))
    checked = (0, 3, 30)
    assert 3 not in host and 0 in host and 30 in host
    O_dec = H.empty_like_storage((L, B, sh.num_q_heads, sh.head_dim), "bf16")
    shared = H.empty_like_storage(Q.shape, "bf16")
    O_pf = [H.empty_like_storage(Q.shape, "bf16") if l in checked else shared for l in range(L)]
    it.run(q_dev, O_dec, lambda l: (Qd, Kd, Vd), O_pf)
    it.finish()
    got = H.to_host(O_dec, "bf16")
    starts = np.concatenate([[0], np.cumsum(dlens)])
    for l in checked:
        for s in (int(np.argmin(dlens)), int(np.argmax(dlens))):
            n = dlens[s]
            o = orc.LayerKVOracle(1, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, bs, wl.blocks_for(n, bs), "bf16")
            o.alloc_layer_blocks(0, 0, n)
            k_l, v_l = kv_of(l)
            o.write_kv(k_l[starts[s]:starts[s] + n], v_l[starts[s]:starts[s] + n], o.slot_mapping(0, 0, 0, n))
            ref = o.paged_decode_attention(q_host[l][s:s + 1], o.padded_block_table([0], 0), [n], threads=THREADS)
            H.check_attention(got[l][s:s + 1], ref, "bf16", scale, f"decode layer {l} sequence {s} ({n} tokens)")
            if l == 30:   # the sequence's stretch of the layer's host image holds the same tokens
                first = sum(wl.blocks_for(m, bs) for m in dlens[:s]) * sh.block_bytes
                mine = it.images[l][first:first + wl.blocks_for(n, bs) * sh.block_bytes].tobytes()
                assert same_tokens(mine, o.pack_layer_blocks(o.block_table(0, 0)).tobytes(), [n], sh), "layer image"
        sampled_prefill_check(5, l, Q, K, V, O_pf[l], plens, sh, scale, [(0, 0), (0, 13), (1, 31), (1, 20)])
    o = orc.LayerKVOracle(1, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, bs, pblk, "bf16")
    for i, n in enumerate(plens):
        o.alloc_layer_blocks(i, 0, n)
    o.write_kv(K, V, np.concatenate([o.slot_mapping(i, 0, 0, n) for i, n in enumerate(plens)]))
    want = o.pack_layer_blocks(sum((o.block_table(i, 0) for i in range(len(plens))), []))
    assert it.prompt_images[0].tobytes() == want.tobytes(), "offload image of the new prompts, layer 0"
    it.close()


# ----------------------------------------------------------------------------- workload 3 as the config is written
def test_workload3_batch_of_four_16k_prompts_offload_reload_and_64_decode_steps():
    """Workload 3 through ``LayerKVEngine`` (the calls ``bench.py`` issues) at its own batch: FOUR 16384-token prompts
    in one launch, three of the 32 layers carried through the whole life cycle: layer 3 is one the even spread of
    Section 3.2.2 retains (24 of 32 offloaded keeps 3, 7, ..., 31), layers 4 and 30 are offloaded (a full 1 GiB image
    each, compared byte for byte), freed, and reloaded into other blocks.  Then all 64 decode steps run on layers 3
    and 30; the oracle checks the steps that open a new block (0 and 16), the one that fills it (15) and the last
    (63): tables bit-exact after every crossing, every output row of the 4 x (16384 + step + 1) split decode.
    The pool holds what these three layers need (the workload's 32 GiB pool adds nothing to the launches)."""
    w = wl.workload(3)
    sh, lens = w.shape, list(w.prompt_lens)
    B, T, bs = len(lens), sum(lens), sh.block_size
    retained = orc.retained_layers(sh.num_layers, sh.num_layers - len(w.offload_layers))
    assert sorted(set(range(sh.num_layers)) - set(retained)) == list(w.offload_layers)
    kept, gone = 3, (4, 30)
    assert kept in retained and all(l in w.offload_layers for l in gone)
    per_layer = sum(wl.blocks_for(n + w.decode_steps, bs) for n in lens)
    nblk = 3 * per_layer + 512
    order = wl.free_list_order(3, nblk, index=7)
    pool = torch.zeros(nblk * sh.block_bytes, dtype=torch.uint8, device=H.DEV)
    eng = LayerKVEngine(sh, nblk, order, pool=pool)
    o = orc.LayerKVOracle(sh.num_layers, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, bs, nblk, sh.dtype)
    o.pool_reset(order)
    eng.begin_prompts(lens)
    layer_bytes = sum(wl.blocks_for(n, bs) for n in lens) * sh.block_bytes
    assert layer_bytes == 1 << 30
    pinned = {l: eng.pinned(layer_bytes) for l in gone}
    for layer in (kept,) + gone:
        Q = wl.normal_tensor_chunked(3, "q", layer, (T, sh.num_q_heads, sh.head_dim), w.data_scale, "bf16")
        K = wl.normal_tensor_chunked(3, "k", layer, (T, sh.num_kv_heads, sh.head_dim), w.data_scale, "bf16")
        V = wl.normal_tensor_chunked(3, "v", layer, (T, sh.num_kv_heads, sh.head_dim), w.data_scale, "bf16")
        Qd, Kd, Vd = H.to_dev(Q), H.to_dev(K), H.to_dev(V)
        Od = H.empty_like_storage(Q.shape, "bf16")
        eng.prefill_layer(layer, Qd, Kd, Vd, Od, offload_to=pinned.get(layer))
        for s, n in enumerate(lens):
            o.alloc_layer_blocks(s, layer, n)
            assert eng.ctx.get_block_table(s, layer).tolist() == o.block_table(s, layer)
        o.write_kv(K, V, np.concatenate([o.slot_mapping(s, layer, 0, n) for s, n in enumerate(lens)]))
        torch.cuda.synchronize()
        # sampled rows of ALL FOUR sequences (two heads each): the work order of a batch of long prompts
        sampled_prefill_check(3, layer, Q, K, V, Od, lens, sh, w.data_scale,
                              [(s, h) for s in range(B) for h in ((5 * s + layer) % 32, 31 - s)], rows_per=40)
        say(f"workload 3: layer {layer} prefilled, sampled rows of four prompts match")
        if layer in gone:
            eng.ctx.event_synchronize(layer, lkv.LKV_EV_OFFLOADED)
            ids = sum((o.block_table(s, layer) for s in range(B)), [])
            assert pinned[layer].numpy().tobytes() == o.pack_layer_blocks(ids).tobytes(), f"offload image, layer {layer}"
        del Q, K, V, Qd, Kd, Vd, Od
    # release both offloaded layers, let someone else take blocks in between, reload into whatever is free now
    old = {l: sum((o.block_table(s, l) for s in range(B)), []) for l in gone}
    for l in gone:
        eng.release_offloaded(l)
        for s in range(B):
            o.free_layer_blocks(s, l, to_host=True)
    eng.ctx.alloc_layer_blocks(999, 0, bs * 100)
    o.alloc_layer_blocks(999, 0, bs * 100)
    for l in gone:
        eng.reload_layer(l)
        for s, n in enumerate(lens):
            o.alloc_layer_blocks(s, l, n)
        new_ids = sum((o.block_table(s, l) for s in range(B)), [])
        assert new_ids != old[l]
        o.unpack_layer_blocks(new_ids, pinned[l].numpy())       # the image was shown equal to the oracle's above
        torch.cuda.synchronize()
        pool_blocks_equal(pool, o, new_ids, f"after reload, layer {l}")
        say(f"workload 3: layer {l} offloaded (1 GiB image equal), reloaded into other blocks")
    # 64 decode steps on the retained layer and on one reloaded layer
    checked_steps = (0, 15, 16, 63)
    for layer in (kept, 30):
        for step in range(w.decode_steps):
            q, k, v = wl.decode_qkv(3, layer, step, B, sh, w.data_scale, q_gain=8.0)
            Od = H.empty_like_storage(q.shape, "bf16")
            eng.decode_layer(layer, H.to_dev(q), H.to_dev(k), H.to_dev(v), Od, step=step)
            slots = []
            for s, n in enumerate(lens):
                o.alloc_layer_blocks(s, layer, n + step + 1)
                slots.append(o.slot_mapping(s, layer, n + step, 1))
            o.write_kv(k, v, np.concatenate(slots))
            if step % bs == 0 or step in checked_steps:       # a new block was opened (steps 0, 16, 32, 48)
                for s in range(B):
                    assert eng.ctx.get_block_table(s, layer).tolist() == o.block_table(s, layer), (layer, step, s)
            if step in checked_steps:
                bt = o.padded_block_table(range(B), layer)
                ref = o.paged_decode_attention(q, bt, [n + step + 1 for n in lens], threads=THREADS)
                torch.cuda.synchronize()
                H.check_attention(H.to_host(Od, "bf16"), ref, "bf16", w.data_scale, f"decode layer {layer} step {step}")
                say(f"workload 3: decode layer {layer} step {step} matches")
        ids = sum((o.block_table(s, layer) for s in range(B)), [])
        assert len(ids) == per_layer
        torch.cuda.synchronize()
        pool_blocks_equal(pool, o, ids, f"after 64 appended tokens, layer {layer}")
    eng.close()


# ----------------------------------------------------------------------------- workload 5 at all 64 sequences
def test_workload5_all_64_decode_sequences_through_the_ring_every_row():
    """The mixed iteration of workload 5 with ALL 64 decoding sequences (contexts 563..16227, 8.8 GiB of KV per
    layer): the launch ``bench.py`` times (2048 (sequence, head) units x 4 partitions, plain work order, not the
    longest-first list of small batches).  Three layers: layer 1 stays on the GPU, layers 0 and 2 live in ordinary
    host memory and come back through a ring of ONE set of blocks (layer 2's reload takes the blocks layer 0's decode
    has just released), the two 8192-token prompts prefill and leave alongside.  Every decode row of every layer is
    compared with the oracle (per sequence: its tokens written into an oracle pool of its own, attended through the
    oracle's table); the new prompts' offload images byte for byte; sampled causal rows of the prompts."""
    from paper_2410_00428_amd.serving import MixedIteration
    w = wl.workload(5)
    bs = w.shape.block_size
    L, host = 3, (0, 2)
    sh = wl.KVShape(L, w.shape.num_q_heads, w.shape.num_kv_heads, w.shape.head_dim, bs, "bf16")
    dlens, plens = list(w.decode_lens), list(w.prompt_lens)
    B, Td, T = len(dlens), sum(dlens), sum(plens)
    assert B == 64
    dblk = sum(wl.blocks_for(n, bs) for n in dlens)
    pblk = sum(wl.blocks_for(n, bs) for n in plens)
    nblk = (L - len(host) + 1) * dblk + L * pblk + 64
    it = MixedIteration(sh, dlens, plens, host, nblk, ring_layers=1, free_order=wl.free_list_order(5, nblk, index=5),
                        tier_unit_bytes=64 << 20, tier_units=4, tier_threads=8)
    scale = w.data_scale
    A = wl.normal_tensor_chunked(5, "k", 950, (Td, sh.num_kv_heads, sh.head_dim), scale, "bf16")
    Bt = wl.normal_tensor_chunked(5, "v", 950, (Td, sh.num_kv_heads, sh.head_dim), scale, "bf16")
    kv_of = lambda l: (A, Bt) if l % 2 == 0 else (Bt, A)
    Ad, Bd = H.to_dev(A), H.to_dev(Bt)
    q_host = [wl.decode_qkv(5, l, 1, B, sh, scale, q_gain=0.25)[0] for l in range(L)]
    q_dev = [H.to_dev(q) for q in q_host]
    Q, K, V = wl.qkv(5, 951, T, sh, scale, q_gain=0.25)
    Qd, Kd, Vd = H.to_dev(Q), H.to_dev(K), H.to_dev(V)
    say("workload 5: inputs drawn and uploaded")
    it.build_cached_state(lambda l: (Ad, Bd) if l % 2 == 0 else (Bd, Ad))
    say("workload 5: cached state built (two layers in host memory)")
    O_dec = H.empty_like_storage((L, B, sh.num_q_heads, sh.head_dim), "bf16")
    O_dec.fill_(0x7FC0)
    O_pf = [H.empty_like_storage(Q.shape, "bf16") for _ in range(L)]
    it.run(q_dev, O_dec, lambda l: (Qd, Kd, Vd), O_pf)
    it.finish()
    got = H.to_host(O_dec, "bf16")
    starts = np.concatenate([[0], np.cumsum(dlens)])
    for s, n in enumerate(dlens):
        o = orc.LayerKVOracle(1, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, bs, wl.blocks_for(n, bs), "bf16")
        o.pool_reset(np.random.default_rng(s).permutation(wl.blocks_for(n, bs)))
        o.alloc_layer_blocks(0, 0, n)
        slots, bt = o.slot_mapping(0, 0, 0, n), o.padded_block_table([0], 0)
        for l in range(L):
            k_l, v_l = kv_of(l)
            o.write_kv(k_l[starts[s]:starts[s] + n], v_l[starts[s]:starts[s] + n], slots)
            ref = o.paged_decode_attention(q_host[l][s:s + 1], bt, [n], threads=THREADS)
            H.check_attention(got[l][s:s + 1], ref, "bf16", scale, f"decode layer {l} sequence {s} ({n} tokens)")
        if s % 8 == 7:
            say(f"workload 5: decode rows of sequences 0..{s} match in all three layers")
    o = orc.LayerKVOracle(1, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, bs, pblk, "bf16")
    for i, n in enumerate(plens):
        o.alloc_layer_blocks(i, 0, n)
    o.write_kv(K, V, np.concatenate([o.slot_mapping(i, 0, 0, n) for i, n in enumerate(plens)]))
    want = o.pack_layer_blocks(sum((o.block_table(i, 0) for i in range(len(plens))), [])).tobytes()
    for l in host:
        assert it.prompt_images[l].tobytes() == want, f"offload image of the new prompts, layer {l}"
        sampled_prefill_check(5, l, Q, K, V, O_pf[l], plens, sh, scale, [(0, 7), (1, 24)], rows_per=32)
    it.close()
