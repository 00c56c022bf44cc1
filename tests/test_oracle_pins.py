"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle itself.

Each test targets a class of plausible mistakes (dropped scale, wrong mask bound, K/V swapped,
wrong head grouping, wrong in-block order, wrong free-list discipline ...).
"""
import os

import numpy as np
import pytest

from oracle import layerkv_oracle as orc
from paper_2410_00428_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers (test-local)
def brute_attention_row(q, Ks, Vs, scale):
    """fp64 textbook softmax attention of one query over explicit key/value lists."""
    logits = [scale * sum(float(a) * float(b) for a, b in zip(q, k)) for k in Ks]
    top = max(logits)
    w = [np.exp(x - top) for x in logits]
    z = sum(w)
    return [sum(w[j] * float(Vs[j][c]) for j in range(len(Ks))) / z for c in range(len(Vs[0]))]


def brute_prefill(Q, K, V, lens, causal, scale):
    T, Hq, d = Q.shape
    Hkv = K.shape[1]
    out = np.zeros((T, Hq, d))
    t0 = 0
    for n in lens:
        for h in range(Hq):
            g = h // (Hq // Hkv)
            for i in range(n):
                last = i + 1 if causal else n
                out[t0 + i, h] = brute_attention_row(Q[t0 + i, h], [K[t0 + j, g] for j in range(last)],
                                                     [V[t0 + j, g] for j in range(last)], scale)
        t0 += n
    return out


def rand(rng, *shape):
    return rng.standard_normal(shape).astype(np.float32)


def build_paged(rng, lens, L=1, Hq=2, Hkv=2, d=8, bs=4, pool_blocks=64, dtype="f32", perm=None):
    o = orc.LayerKVOracle(L, Hq, Hkv, d, bs, pool_blocks, dtype)
    o.pool_reset(perm if perm is not None else rng.permutation(pool_blocks))
    data = {}
    for layer in range(L):
        for s, n in enumerate(lens):
            o.alloc_layer_blocks(s, layer, n)
            K, V = rand(rng, n, Hkv, d), rand(rng, n, Hkv, d)
            if dtype == "bf16":
                K, V = wl.f32_to_bf16_bits(K), wl.f32_to_bf16_bits(V)
            o.write_kv(K, V, o.slot_mapping(s, layer, 0, n))
            data[(s, layer)] = (K, V)
    return o, data


# ----------------------------------------------------------------------------- attention vs brute force
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2), (4, 1)])
def test_prefill_matches_bruteforce(causal, Hq, Hkv):
    rng = np.random.default_rng(1)
    lens, d = (5, 33), 8
    T = sum(lens)
    Q, K, V = rand(rng, T, Hq, d), rand(rng, T, Hkv, d), rand(rng, T, Hkv, d)
    scale = 0.37  # deliberately not 1/sqrt(d): catches an ignored scale argument
    got = orc.prefill_attention(Q, K, V, wl.cu_seqlens(lens), "f32", causal=causal, scale=scale)
    ref = brute_prefill(Q, K, V, lens, causal, scale)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_default_scale_is_inverse_sqrt_head_dim():
    rng = np.random.default_rng(2)
    Q, K, V = rand(rng, 9, 1, 16), rand(rng, 9, 1, 16), rand(rng, 9, 1, 16)
    got = orc.prefill_attention(Q, K, V, [0, 9], "f32")
    ref = brute_prefill(Q, K, V, (9,), True, 16 ** -0.5)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_prefill_matches_library_sdpa():
    """Same numbers as torch's scaled_dot_product_attention on CPU in float64."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(3)
    n, Hq, Hkv, d = 77, 4, 2, 32
    Q, K, V = rand(rng, n, Hq, d), rand(rng, n, Hkv, d), rand(rng, n, Hkv, d)
    got = orc.prefill_attention(Q, K, V, [0, n], "f32", causal=True)
    q = torch.from_numpy(Q).double().permute(1, 0, 2)[None]
    k = torch.from_numpy(K).double().permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    v = torch.from_numpy(V).double().permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)


def test_paged_decode_matches_bruteforce():
    rng = np.random.default_rng(4)
    lens = (1, 4, 7, 13)
    o, data = build_paged(rng, lens, Hq=4, Hkv=2, d=8, bs=4)
    Q = rand(rng, len(lens), 4, 8)
    bt = o.padded_block_table(range(len(lens)), 0)
    got = o.paged_decode_attention(Q, bt, lens, scale=0.5)
    for s, n in enumerate(lens):
        K, V = data[(s, 0)]
        for h in range(4):
            ref = brute_attention_row(Q[s, h], [K[j, h // 2] for j in range(n)], [V[j, h // 2] for j in range(n)], 0.5)
            np.testing.assert_allclose(got[s, h], ref, rtol=1e-12, atol=1e-13)


def test_sampled_rows_equal_full_result():
    rng = np.random.default_rng(5)
    lens = (19, 40)
    T, Hq, Hkv, d = sum(lens), 4, 2, 16
    Q, K, V = rand(rng, T, Hq, d), rand(rng, T, Hkv, d), rand(rng, T, Hkv, d)
    cu = wl.cu_seqlens(lens)
    full = orc.prefill_attention(Q, K, V, cu, "f32")
    tok = np.array([0, 18, 19, 35, 58])
    head = np.array([0, 3, 1, 2, 3], dtype=np.int32)
    rows = orc.prefill_attention_rows(Q, K, V, cu, "f32", tok, head)
    for r in range(len(tok)):
        assert np.array_equal(rows[r], full[tok[r], head[r]])


# ----------------------------------------------------------------------------- closed forms
def test_equal_keys_give_prefix_mean_of_values():
    rng = np.random.default_rng(6)
    n, d = 23, 8
    K = np.repeat(rand(rng, 1, 1, d), n, axis=0)
    Q, V = rand(rng, n, 1, d), rand(rng, n, 1, d)
    got = orc.prefill_attention(Q, K, V, [0, n], "f32")[:, 0]
    ref = np.cumsum(V[:, 0].astype(np.float64), axis=0) / np.arange(1, n + 1)[:, None]
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-14)


def test_constant_values_come_back_unchanged_and_row0_is_v0():
    rng = np.random.default_rng(7)
    n, d = 31, 8
    Q, K = rand(rng, n, 2, d), rand(rng, n, 2, d)
    V = np.tile(rand(rng, 1, 2, d), (n, 1, 1))
    got = orc.prefill_attention(Q, K, V, [0, n], "f32")
    np.testing.assert_allclose(got, np.broadcast_to(V[0], got.shape).astype(np.float64), rtol=1e-13)
    V2 = rand(rng, n, 2, d)
    got2 = orc.prefill_attention(Q, K, V2, [0, n], "f32")
    assert np.array_equal(got2[0], V2[0].astype(np.float64))


def test_dominant_logit_selects_its_value():
    n, d = 12, 4
    K = np.zeros((n, 1, d), np.float32)
    K[5, 0, 0] = 60.0
    Q = np.zeros((n, 1, d), np.float32)
    Q[:, 0, 0] = 1.0
    V = np.arange(n * d, dtype=np.float32).reshape(n, 1, d)
    got = orc.prefill_attention(Q, K, V, [0, n], "f32", causal=False, scale=1.0)
    np.testing.assert_allclose(got[:, 0], np.broadcast_to(V[5, 0], (n, d)), rtol=0, atol=1e-20 * 50)


def test_softmax_shift_invariance():
    """Adding one vector to every key shifts all logits of a row equally: output unchanged."""
    rng = np.random.default_rng(8)
    n, d = 17, 8
    Q, V = rand(rng, n, 1, d), rand(rng, n, 1, d)
    K = np.round(rand(rng, n, 1, d) * 8) / 8          # multiples of 1/8: K + c is exact in float32
    c = np.round(rand(rng, 1, 1, d) * 8) / 8
    a = orc.prefill_attention(Q, K.astype(np.float32), V, [0, n], "f32")
    b = orc.prefill_attention(Q, (K + c).astype(np.float32), V, [0, n], "f32")
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)


def test_zero_context_gives_zero_row():
    rng = np.random.default_rng(9)
    o, _ = build_paged(rng, (6,), Hq=2, Hkv=2)
    Q = rand(rng, 1, 2, 8)
    got = o.paged_decode_attention(Q, o.padded_block_table([0], 0), [0])
    assert np.array_equal(got, np.zeros_like(got))


# ----------------------------------------------------------------------------- paging invariants
def test_paged_equals_dense_on_gathered_kv_and_decode_equals_last_prefill_row():
    rng = np.random.default_rng(10)
    lens = (9, 16, 30)
    o, data = build_paged(rng, lens, Hq=4, Hkv=2, d=8, bs=4)
    for s, n in enumerate(lens):
        Kg, Vg = o.gather_layer_kv(s, 0, n)
        assert np.array_equal(Kg, data[(s, 0)][0]) and np.array_equal(Vg, data[(s, 0)][1])
        Q = rand(rng, n, 4, 8)
        dense = orc.prefill_attention(Q, Kg, Vg, [0, n], "f32")
        paged = o.paged_decode_attention(Q[n - 1:n], o.padded_block_table([s], 0), [n])
        assert np.array_equal(paged[0], dense[n - 1])  # same order of operations: bit-identical


def test_result_does_not_depend_on_physical_block_ids():
    lens = (9, 16, 30)
    outs = []
    for perm_seed in (0, 1):
        rng = np.random.default_rng(11)  # same data both times
        perm = np.random.default_rng(100 + perm_seed).permutation(64)
        o, _ = build_paged(rng, lens, Hq=2, Hkv=2, perm=perm)
        Q = rand(np.random.default_rng(12), len(lens), 2, 8)
        outs.append(o.paged_decode_attention(Q, o.padded_block_table(range(3), 0), lens))
    assert np.array_equal(outs[0], outs[1])


def test_every_layer_has_its_own_table():
    rng = np.random.default_rng(13)
    o, data = build_paged(rng, (10, 7), L=3, Hq=2, Hkv=2)
    tabs = [o.block_table(0, l) for l in range(3)]
    assert len({tuple(t) for t in tabs}) == 3 and not set(tabs[0]) & set(tabs[1])
    for l in range(3):
        Kg, Vg = o.gather_layer_kv(0, l, 10)
        assert np.array_equal(Kg, data[(0, l)][0])


def test_unused_slots_and_stale_blocks_do_not_leak():
    rng = np.random.default_rng(14)
    o, _ = build_paged(rng, (5, 9), Hq=2, Hkv=2)
    Q = rand(rng, 2, 2, 8)
    bt = o.padded_block_table([0, 1], 0)
    clean = o.paged_decode_attention(Q, bt, [5, 9])
    used = {(b, off) for s, n in ((0, 5), (1, 9)) for b, off in
            (divmod(int(x), o.bs) for x in o.slot_mapping(s, 0, 0, n))}
    for b in range(o.num_pool_blocks):
        for off in range(o.bs):
            if (b, off) not in used:
                o.pool[b, :, :, off, :] = np.nan
    assert np.array_equal(o.paged_decode_attention(Q, bt, [5, 9]), clean)
    assert np.isfinite(clean).all()


def test_gqa_equals_mha_with_repeated_kv_heads():
    rng = np.random.default_rng(15)
    n, Hq, Hkv, d = 21, 8, 2, 8
    Q, K, V = rand(rng, n, Hq, d), rand(rng, n, Hkv, d), rand(rng, n, Hkv, d)
    a = orc.prefill_attention(Q, K, V, [0, n], "f32")
    b = orc.prefill_attention(Q, np.repeat(K, 4, axis=1), np.repeat(V, 4, axis=1), [0, n], "f32")
    assert np.array_equal(a, b)


# ----------------------------------------------------------------------------- storage format
def test_write_lands_at_documented_byte_offsets():
    """Block b at b*beta; inside: [kv head][K|V][token][channel] -- the format lkv.h documents."""
    rng = np.random.default_rng(16)
    Hkv, d, bs = 3, 8, 4
    o = orc.LayerKVOracle(1, 3, Hkv, d, bs, 16, "f32")
    o.pool_reset(rng.permutation(16))
    o.alloc_layer_blocks(0, 0, 10)
    K, V = rand(rng, 10, Hkv, d), rand(rng, 10, Hkv, d)
    slots = o.slot_mapping(0, 0, 0, 10)
    o.write_kv(K, V, slots)
    flat = o.pool.reshape(-1)
    for t in range(10):
        b, off = divmod(int(slots[t]), bs)
        for h in range(Hkv):
            base = b * (Hkv * 2 * bs * d) + h * (2 * bs * d) + off * d
            assert np.array_equal(flat[base:base + d], K[t, h])
            assert np.array_equal(flat[base + bs * d:base + bs * d + d], V[t, h])


def test_negative_slot_skips_token():
    o = orc.LayerKVOracle(1, 1, 1, 4, 2, 4, "f32")
    K = np.ones((2, 1, 4), np.float32)
    o.write_kv(K, K, np.array([-1, 3]))
    assert o.pool.sum() == 8 and o.pool[1, 0, :, 1, :].sum() == 8


def test_pack_then_unpack_is_identity_even_into_other_blocks():
    rng = np.random.default_rng(17)
    lens = (11, 6)
    o, data = build_paged(rng, lens, L=2, Hq=2, Hkv=2)
    Q = rand(rng, 2, 2, 8)
    before = o.paged_decode_attention(Q, o.padded_block_table([0, 1], 1), lens)
    images, old = {}, {}
    for s in (0, 1):
        ids = o.block_table(s, 1)
        old[s] = ids
        images[s] = o.pack_layer_blocks(ids).copy()
        assert images[s].nbytes == len(ids) * o.pool[0].nbytes
        for i, b in enumerate(ids):  # brute-force byte check of the image
            assert images[s][i * o.pool[0].nbytes:(i + 1) * o.pool[0].nbytes].tobytes() == o.pool[b].tobytes()
        o.free_layer_blocks(s, 1, to_host=True)
        assert o.layer_residency(s, 1) == orc.HOST
    o.pool[:] = np.where(np.isin(np.arange(o.num_pool_blocks), old[0] + old[1])[:, None, None, None, None], np.nan, o.pool)
    # occupy some blocks so the reload lands elsewhere
    o.alloc_layer_blocks(99, 0, 8)
    for s in (1, 0):
        o.alloc_layer_blocks(s, 1, lens[s])
        o.unpack_layer_blocks(o.block_table(s, 1), images[s])
        assert o.layer_residency(s, 1) == orc.GPU
    assert o.block_table(0, 1) != old[0]
    for s in (0, 1):
        Kg, Vg = o.gather_layer_kv(s, 1, lens[s])
        assert np.array_equal(Kg, data[(s, 1)][0]) and np.array_equal(Vg, data[(s, 1)][1])
    after = o.paged_decode_attention(Q, o.padded_block_table([0, 1], 1), lens)
    assert np.array_equal(before, after)


# ----------------------------------------------------------------------------- allocator / tables
def test_slot_mapping_is_injective_and_inside_owned_blocks():
    rng = np.random.default_rng(18)
    o, _ = build_paged(rng, (13, 4, 8), L=2, Hq=2, Hkv=2)
    seen = set()
    for layer in range(2):
        for s, n in enumerate((13, 4, 8)):
            for p, slot in enumerate(o.slot_mapping(s, layer, 0, n)):
                assert slot // o.bs == o.block_table(s, layer)[p // o.bs] and slot % o.bs == p % o.bs
                assert slot not in seen
                seen.add(int(slot))


def test_allocator_replays_a_lifo_model_and_conserves_blocks():
    """Independent ten-line model: a stack; alloc pops, free pushes the table in order."""
    rng = np.random.default_rng(19)
    N, bs = 40, 4
    o = orc.LayerKVOracle(3, 1, 1, 4, bs, N, "f32")
    order = rng.permutation(N)
    o.pool_reset(order)
    stack, tabs = list(order[::-1]), {}
    for step in range(400):
        seq, layer = int(rng.integers(0, 5)), int(rng.integers(0, 3))
        if rng.random() < 0.6:
            n = int(rng.integers(0, 30))
            want = max(-(-n // bs), len(tabs.get((seq, layer), [])))
            grow = want - len(tabs.get((seq, layer), []))
            if grow > len(stack):
                with pytest.raises(orc.NoBlocks):
                    o.alloc_layer_blocks(seq, layer, n)
            else:
                o.alloc_layer_blocks(seq, layer, n)
                tabs.setdefault((seq, layer), [])
                for _ in range(grow):
                    tabs[(seq, layer)].append(int(stack.pop()))
        elif (seq, layer) in tabs:
            o.free_layer_blocks(seq, layer)
            stack.extend(tabs.pop((seq, layer)))
        assert o.block_table(seq, layer) == tabs.get((seq, layer), [])
        assert o.num_free_blocks() + sum(len(t) for t in o.tables.values()) == N
        assert o.num_free_blocks() == len(stack)
    first = orc.LayerKVOracle(1, 1, 1, 4, bs, 8, "f32")
    first.pool_reset([5, 2, 7, 0, 1, 3, 4, 6])
    first.alloc_layer_blocks(0, 0, 9)
    assert first.block_table(0, 0) == [5, 2, 7]  # free_order[0] is handed out first


def test_free_seq_releases_everything():
    o = orc.LayerKVOracle(4, 1, 1, 4, 4, 32, "f32")
    for l in range(4):
        o.alloc_layer_blocks(7, l, 10)
    o.alloc_layer_blocks(8, 0, 4)
    o.free_seq(7)
    assert o.num_free_blocks() == 31 and o.block_table(7, 2) == []


def test_free_seq_release_order_replays_the_stack_model():
    """A finished request gives its layers back lowest layer first, each table in table order, onto the stack: the
    ids handed out next are the LAST layer's table read backwards, then the layer before it, and so on.  Checked
    against an independent list model, with another request's blocks in between."""
    N, bs, L = 24, 4, 3
    order = [int(v) for v in np.random.default_rng(31).permutation(N)]
    o = orc.LayerKVOracle(L, 1, 1, 4, bs, N, "f32")
    o.pool_reset(order)
    stack = order[::-1]
    tabs = {}
    for seq, layer, tokens in ((7, 0, 9), (8, 1, 5), (7, 2, 4), (7, 1, 13), (8, 0, 1)):
        o.alloc_layer_blocks(seq, layer, tokens)
        tabs[(seq, layer)] = [stack.pop() for _ in range(-(-tokens // bs))]
        assert o.block_table(seq, layer) == tabs[(seq, layer)]
    t70, t71, t72 = tabs[(7, 0)], tabs[(7, 1)], tabs[(7, 2)]       # 3, 4 and 1 blocks
    o.free_seq(7)
    for layer in range(L):                      # the model: lowest layer first, each table in table order
        stack.extend(tabs.pop((7, layer)))
    assert o.num_free_blocks() == len(stack)
    assert [o.layer_residency(7, l) for l in range(L)] == [None] * L
    # the stack hands out the last layer's blocks first, each table backwards: written out, not derived
    o.alloc_layer_blocks(9, 0, 8 * bs)
    assert o.block_table(9, 0) == t72[::-1] + t71[::-1] + t70[::-1]
    assert o.block_table(9, 0) == [stack.pop() for _ in range(8)]
    assert o.block_table(8, 1) == tabs[(8, 1)] and o.block_table(8, 0) == tabs[(8, 0)]   # the other request: untouched


def test_retained_layers_matches_the_papers_example():
    txt = dict(line.split(None, 1) for line in open(os.path.join(GOLDEN, "retained_layers_L8_x4.txt"))
               if not line.startswith("#"))
    L, x = int(txt["num_layers"]), int(txt["retained_count"])
    keep = orc.retained_layers(L, x)
    assert keep == [int(v) for v in txt["retained"].split()]
    assert [l for l in range(L) if l not in keep] == [int(v) for v in txt["offloaded"].split()]
    for L in (8, 32, 80):
        for x in range(L + 1):
            k = orc.retained_layers(L, x)
            assert len(k) == x and k == sorted(set(k))
            if 0 < x < L:  # evenly spread: gaps differ by at most one
                gaps = np.diff([-1] + k) if False else np.diff(k + [k[0] + L])
                assert gaps.max() - gaps.min() <= 1


# ----------------------------------------------------------------------------- precision
def test_fp32_accumulation_stays_within_rounding_bound_of_fp64():
    rng = np.random.default_rng(20)
    n, d = 512, 64
    Q, K, V = rand(rng, n, 1, d), rand(rng, n, 1, d), rand(rng, n, 1, d)
    a = orc.prefill_attention(Q, K, V, [0, n], "f32", acc="f64")
    b = orc.prefill_attention(Q, K, V, [0, n], "f32", acc="f32")
    rowmax = np.abs(a).max(axis=-1, keepdims=True)
    assert (np.abs(a - b) <= 4 * n * 2.0 ** -24 * rowmax).all()
    assert not np.array_equal(a, b)


def test_bf16_inputs_are_widened_exactly():
    rng = np.random.default_rng(21)
    n, d = 19, 16
    Qb, Kb, Vb = (wl.f32_to_bf16_bits(rand(rng, n, 2, d)) for _ in range(3))
    a = orc.prefill_attention(Qb, Kb, Vb, [0, n], "bf16")
    b = orc.prefill_attention(wl.bf16_bits_to_f32(Qb), wl.bf16_bits_to_f32(Kb), wl.bf16_bits_to_f32(Vb), [0, n], "f32")
    assert np.array_equal(a, b)


def test_bf16_rounding_helper_is_round_to_nearest_even():
    torch = pytest.importorskip("torch")
    x = np.random.default_rng(22).standard_normal(4096).astype(np.float32)
    x[:4] = [1.0, 1.00390625, 1.01171875, -0.0]  # exact, tie-to-even down, tie-to-even up, signed zero
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(wl.f32_to_bf16_bits(x), ref)
    assert np.array_equal(wl.bf16_bits_to_f32(ref), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_multithreaded_run_is_bit_identical():
    rng = np.random.default_rng(23)
    lens = (40, 25)
    T = sum(lens)
    Q, K, V = rand(rng, T, 4, 16), rand(rng, T, 2, 16), rand(rng, T, 2, 16)
    a = orc.prefill_attention(Q, K, V, wl.cu_seqlens(lens), "f32", threads=1)
    b = orc.prefill_attention(Q, K, V, wl.cu_seqlens(lens), "f32", threads=4)
    assert np.array_equal(a, b)
