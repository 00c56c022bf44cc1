"""GPU parity of one mixed serving iteration (``paper_2410_00428_amd.serving.MixedIteration``: what
``bench.py --workload 5`` times at full size) against the oracle, at a size the oracle finishes in seconds: host
layers of the decode batch in ordinary host memory, reloaded through a two-layer ring of blocks while the new
prompts prefill and leave.  The oracle keeps every layer in its own pool under its own block ids: attention
results, block contents and offload images do not depend on which blocks hold them (Section 3.2.2)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import layerkv_oracle as orc  # noqa: E402
from paper_2410_00428_amd import workloads as wl  # noqa: E402
from paper_2410_00428_amd.serving import MixedIteration  # noqa: E402
from tests import gpu_harness as H  # noqa: E402

pytestmark = pytest.mark.gpu
THREADS = 16


def same_tokens(a, b, lens, sh) -> bool:
    """Two images of the same sequences' blocks (sequence after sequence) hold the same bytes at every cached token.
    The slots behind a sequence's last token are not compared: a block that held another layer before keeps that
    layer's bytes there, and nothing ever reads them."""
    shape5 = (-1, sh.num_kv_heads, 2, sh.block_size, sh.head_dim)
    elem = np.uint8 if sh.dtype == "fp8" else np.uint16
    a = np.frombuffer(a, dtype=elem).reshape(shape5)
    b = np.frombuffer(b, dtype=elem).reshape(shape5)
    if a.shape != b.shape:
        return False
    off = 0
    for n in lens:
        full, rest = divmod(n, sh.block_size)
        if not np.array_equal(a[off:off + full], b[off:off + full]):
            return False
        if rest and not np.array_equal(a[off + full, :, :, :rest], b[off + full, :, :, :rest]):
            return False
        off += wl.blocks_for(n, sh.block_size)
    return off == a.shape[0]


@pytest.mark.parametrize("ring,unit_blocks,units,threads,dtype", [(2, 8, 3, 2, "bf16"), (1, 1, 1, 1, "bf16"),
                                                                  (3, 64, 8, 4, "bf16"), (2, 8, 3, 2, "fp8")])
def test_mixed_iteration_host_layers_through_a_ring_of_blocks_and_the_pageable_tier(ring, unit_blocks, units, threads,
                                                                                    dtype):
    sh = wl.KVShape(6, 8, 4, 128, 16, dtype)
    scales = dict(k_scale=1 / 32, v_scale=1 / 64) if dtype == "fp8" else {}
    L, bs = sh.num_layers, sh.block_size
    dlens = [37, 500, 1200, 64, 333, 1999, 16]
    plens = [300, 170]
    B, P, Td, T = len(dlens), len(plens), sum(dlens), sum(plens)
    retained = orc.retained_layers(L, 2)
    host = [l for l in range(L) if l not in retained]
    assert retained == [2, 5]
    dblk = sum(wl.blocks_for(n, bs) for n in dlens)
    pblk = sum(wl.blocks_for(n, bs) for n in plens)
    nblk = (len(retained) + ring) * dblk + L * pblk + 8   # retained layers + the ring + the prompts
    order = wl.free_list_order(5, nblk, index=9)
    pool = H.zero_pool(sh, nblk)
    it = MixedIteration(sh, dlens, plens, host, nblk, ring_layers=ring, free_order=order, pool=pool,
                        tier_unit_bytes=unit_blocks * sh.block_bytes, tier_units=units, tier_threads=threads, **scales)
    c = it.ctx
    o = orc.LayerKVOracle(L, sh.num_q_heads, sh.num_kv_heads, sh.head_dim, bs, L * (dblk + pblk), dtype, **scales)
    scale = 0.5
    kv, qd, pq = {}, [], {}
    for l in range(L):
        kv[l] = tuple(wl.normal_tensor(wl.rng_for(5, n, 300 + l), (Td, sh.num_kv_heads, sh.head_dim), scale, "bf16")
                      for n in ("k", "v"))
        qd.append(wl.normal_tensor(wl.rng_for(5, "q", 300 + l), (B, sh.num_q_heads, sh.head_dim), scale, "bf16"))
        pq[l] = tuple(wl.normal_tensor(wl.rng_for(5, n, 400 + l), (T, h, sh.head_dim), scale, "bf16")
                      for n, h in (("q", sh.num_q_heads), ("k", sh.num_kv_heads), ("v", sh.num_kv_heads)))
        for s, n in enumerate(dlens):
            o.alloc_layer_blocks(s, l, n)
        o.write_kv(kv[l][0], kv[l][1], np.concatenate([o.slot_mapping(s, l, 0, n) for s, n in enumerate(dlens)]))
        for i, n in enumerate(plens):
            o.alloc_layer_blocks(B + i, l, n)
        o.write_kv(pq[l][1], pq[l][2], np.concatenate([o.slot_mapping(B + i, l, 0, n) for i, n in enumerate(plens)]))

    def o_ids(seqs, l):
        return sum((o.block_table(s, l) for s in seqs), [])

    def blocks_of(ids):
        return pool.view(nblk, -1)[torch.from_numpy(np.asarray(ids, dtype=np.int64)).to(H.DEV)].cpu().numpy().tobytes()

    it.build_cached_state(lambda l: (H.to_dev(kv[l][0]), H.to_dev(kv[l][1])))
    torch.cuda.synchronize()
    for l in host:
        same = same_tokens(it.images[l].tobytes(), o.pack_layer_blocks(o_ids(range(B), l)).tobytes(), dlens, sh)
        assert same, f"host image of layer {l}"
        assert c.layer_residency(0, l) == 2
    free_before = c.num_free_blocks()
    assert free_before == nblk - len(retained) * dblk

    q_dev = [H.to_dev(q) for q in qd]
    p_dev = {l: tuple(H.to_dev(a) for a in pq[l]) for l in range(L)}
    first = None
    for rep in range(2):
        O_dec = H.empty_like_storage((L,) + qd[0].shape, "bf16")
        O_pf = [H.empty_like_storage(pq[0][0].shape, "bf16") for _ in range(L)]
        it.run(q_dev, O_dec, lambda l: p_dev[l], O_pf)
        it.finish()
        got_dec = H.to_host(O_dec, "bf16")
        for l in range(L):
            ref = o.paged_decode_attention(qd[l], o.padded_block_table(range(B), l), dlens, threads=THREADS)
            H.check_attention(got_dec[l], ref, "bf16", scale, f"pass {rep}: decode attention, layer {l}")
            refp = orc.prefill_attention(pq[l][0], pq[l][1], pq[l][2], wl.cu_seqlens(plens), "bf16", threads=THREADS)
            H.check_attention(H.to_host(O_pf[l], "bf16"), refp, "bf16", scale, f"pass {rep}: prefill, layer {l}")
        for l in host:      # the new prompts' KV of the host layers is in host memory, the blocks are free again
            want = o.pack_layer_blocks(o_ids(range(B, B + P), l)).tobytes()
            assert same_tokens(it.prompt_images[l].tobytes(), want, plens, sh), f"pass {rep}: new prompts' image, layer {l}"
            assert c.layer_residency(0, l) == 2 and c.layer_residency(B, l) == 2
        for l in retained:  # retained layers: the same bytes in the pool, under the library's own block ids
            ids = np.concatenate([c.get_block_table(s, l) for s in range(B + P)])
            same = same_tokens(blocks_of(ids), o.pool[np.asarray(o_ids(range(B + P), l))].tobytes(), dlens + plens, sh)
            assert same, f"pass {rep}: pool blocks, layer {l}"
        assert c.num_free_blocks() == free_before - len(retained) * pblk
        it.drop_prompts()
        assert c.num_free_blocks() == free_before
        if first is None:
            first = got_dec.copy()
        else:   # other blocks held the reloaded layers this time: the results do not depend on the block ids
            assert got_dec.tobytes() == first.tobytes()
    it.close()
