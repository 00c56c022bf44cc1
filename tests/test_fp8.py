"""The 8-bit KV-cache format (OCP E4M3, the paper's Future Work made concrete): pins of the oracle's codec, then
the library against it."""
from fractions import Fraction as F

import numpy as np
import pytest

from oracle import fp8_codec as fp8
from paper_2410_00428_amd import workloads as wl

torch = pytest.importorskip("torch")


# ----------------------------------------------------------------------------- oracle pins
def test_published_constants_of_the_format():
    """OCP 8-bit floating point specification, E4M3: bias 7, max 448 = S.1111.110, min normal 2^-6, min subnormal
    2^-9, 1.0 = 0.0111.000, no infinities, S.1111.111 is NaN."""
    assert fp8.decode_one(0x7E) == 448 and fp8.decode_one(0xFE) == -448
    assert fp8.decode_one(0x08) == F(1, 64) and fp8.decode_one(0x01) == F(1, 512) and fp8.decode_one(0x07) == F(7, 512)
    assert fp8.decode_one(0x38) == 1 and fp8.decode_one(0x40) == 2 and fp8.decode_one(0x3C) == F(3, 2)
    assert fp8.decode_one(0x00) == 0 and fp8.decode_one(0x80) == 0
    assert fp8.decode_one(0x7F) is None and fp8.decode_one(0xFF) is None
    assert fp8.decode_one(0x78) == 256          # the top exponent holds finite values (no infinities)
    assert all(a < b for a, b in zip(fp8.POSITIVE, fp8.POSITIVE[1:]))


def test_encode_inverts_decode_and_rounds_midpoints_to_even():
    for c in range(256):
        v = fp8.decode_one(c)
        if v is None:
            continue
        want = c if v != 0 else (c & 0x80)
        assert fp8.encode_one(v) == (want if v != 0 or c == 0 else 0)   # -0 as an exact rational is +0
    for i in range(0x7E):
        lo, hi = fp8.POSITIVE[i], fp8.POSITIVE[i + 1]
        mid = (lo + hi) / 2
        even = i if i % 2 == 0 else i + 1
        assert fp8.encode_one(mid) == even and fp8.encode_one(-mid) == (0x80 | even)
        eps = (hi - lo) / 1024
        assert fp8.encode_one(mid - eps) == i and fp8.encode_one(mid + eps) == i + 1
    assert fp8.encode_one(F(1, 1024)) == 0          # half of the smallest subnormal: tie, to even (zero)
    assert fp8.encode_one(F(1, 1024) + F(1, 2**20)) == 1
    assert fp8.encode_one(F(10**6)) == 0x7E and fp8.encode_one(F(-10**6)) == 0xFE     # saturation, not NaN
    assert fp8.encode_one(F(464)) == 0x7E           # past the last midpoint there is nothing to round up to


def test_codec_agrees_with_an_independent_library_conversion():
    """torch's float8_e4m3fn casts (CPU) are a separate implementation of the same format: every float32 that the
    library quantises - a bf16 value times a float32 factor - must get the same code wherever |x| stays inside the
    finite range (torch turns overflow into NaN where this codec saturates: a choice, checked separately)."""
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 2**16, size=20000, dtype=np.uint16)
    with np.errstate(invalid="ignore", over="ignore"):
        x = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32) * np.float32(0.37)
    x = x[np.isfinite(x) & (np.abs(x) <= 448)]
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = fp8.encode(x)
    same = (got == want) | ((x == 0) & ((got & 0x7F) == 0) & ((want & 0x7F) == 0))
    assert same.all()
    codes = np.arange(256, dtype=np.uint8)
    back = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    ours = fp8.decode(codes)
    assert np.array_equal(np.isnan(back), np.isnan(ours)) and np.array_equal(back[~np.isnan(back)], ours[~np.isnan(ours)])


def test_quantize_applies_one_float32_multiply():
    bits = np.array([0x3F80, 0xBF80, 0x4000, 0x3E80, 0x0000, 0x8000, 0x7F80, 0xFF80, 0x4780], dtype=np.uint16)
    # 1, -1, 2, 0.25, 0, -0, inf, -inf, 65536 at scale 0.5: x / 0.5 = 2, -2, 4, 0.5, 0, -0, saturate ...
    assert fp8.quantize_bf16_bits(bits, 0.5).tolist() == [0x40, 0xC0, 0x48, 0x30, 0x00, 0x80, 0x7E, 0xFE, 0x7E]
    # a scale whose reciprocal is inexact: the product is rounded once to float32 before the code is chosen
    x = np.float32(1.0) * (np.float32(1.0) / np.float32(3.0))
    assert fp8.quantize_bf16_bits(np.array([0x3F80], np.uint16), 3.0)[0] == fp8.encode_one(F(float(x)))


def test_reciprocal_product_and_exact_division_are_two_readings_that_differ_at_midpoints():
    """The paper fixes no format, so the quantisation step is a reading: the contract multiplies by the float32
    reciprocal of the scale.  1.3671875 / 7 = 0.1953125 is EXACTLY half way between the codes 0x24 (0.1875) and 0x25
    (0.203125): exact division rounds the tie to the even code 0x24, while fl32(1/7) lies a little above 1/7 and the
    product a little above the midpoint, which gives 0x25.  Away from such midpoints the two agree."""
    x = np.array([0x3FAF], dtype=np.uint16)                       # 1.3671875 as bf16
    assert F(float(wl.bf16_bits_to_f32(x)[0])) / 7 == (fp8.POSITIVE[0x24] + fp8.POSITIVE[0x25]) / 2
    assert fp8.quantize_bf16_bits_exact_division(x, 7.0)[0] == 0x24
    assert fp8.quantize_bf16_bits(x, 7.0)[0] == 0x25
    # powers of two have exact reciprocals: no difference anywhere, midpoints included
    every = np.arange(0x3C00, 0x4400, dtype=np.uint16)
    for scale in (0.5, 4.0):
        assert np.array_equal(fp8.quantize_bf16_bits(every, scale), fp8.quantize_bf16_bits_exact_division(every, scale))
    # an inexact reciprocal: the readings part on a few patterns only, all of them within one code of each other
    a, b = fp8.quantize_bf16_bits(every, 7.0), fp8.quantize_bf16_bits_exact_division(every, 7.0)
    diff = np.flatnonzero(a != b)
    assert 0 < len(diff) < len(every) // 20 and (np.abs(a[diff].astype(int) - b[diff].astype(int)) == 1).all()


def test_oracle_fp8_pool_decode_equals_decode_over_the_dequantised_values():
    """The fp8 oracle is the bf16 one fed with the values the codes stand for: with scales that are powers of two
    and data that the format holds exactly, both give the same result bit for bit; and the offload image is one
    byte per element."""
    from oracle import layerkv_oracle as orc
    rng = np.random.default_rng(3)
    Hq, Hkv, d, bs, n = 4, 2, 128, 16, 70
    grid = np.array([float(v) for v in fp8.POSITIVE[0x20:0x50]], dtype=np.float32)      # values E4M3 holds exactly
    def draw(shape):
        x = rng.choice(grid, size=shape) * rng.choice([-1.0, 1.0], size=shape)
        return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)   # exact in bf16
    K, V = draw((n, Hkv, d)), draw((n, Hkv, d))
    q = draw((1, Hq, d))
    a = orc.LayerKVOracle(1, Hq, Hkv, d, bs, 8, "fp8", k_scale=0.5, v_scale=4.0)
    b = orc.LayerKVOracle(1, Hq, Hkv, d, bs, 8, "bf16")
    for o in (a, b):
        o.alloc_layer_blocks(0, 0, n)
    slots = a.slot_mapping(0, 0, 0, n)
    # a stores K/0.5 and V/4 as codes: give it data pre-multiplied so that both pools stand for the same values
    def times(bits, f):
        x = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32) * np.float32(f)
        return (x.view(np.uint32) >> 16).astype(np.uint16)
    a.write_kv(times(K, 0.5), times(V, 4.0), slots)
    b.write_kv(times(K, 0.5), times(V, 4.0), slots)
    bt = a.padded_block_table([0], 0)
    ra = a.paged_decode_attention(q, bt, [n])
    rb = b.paged_decode_attention(q, bt, [n])
    assert np.allclose(ra, rb, rtol=1e-12, atol=1e-12)
    assert a.pack_layer_blocks(a.block_table(0, 0)).nbytes * 2 == b.pack_layer_blocks(b.block_table(0, 0)).nbytes


# ----------------------------------------------------------------------------- library against the oracle (GPU)
def _fp8_pair(Hq, Hkv, lens, k_scale, v_scale, seed, **kw):
    from paper_2410_00428_amd import workloads as wl
    from tests import gpu_harness as H
    shape = wl.KVShape(1, Hq, Hkv, 128, 16, "fp8")
    nblk = sum((n + 16) // 16 + 1 for n in lens) + 8
    c, o, pool = H.make_pair(shape, nblk, wl.free_list_order(seed, nblk), k_scale=k_scale, v_scale=v_scale, **kw)
    return shape, c, o, pool


@pytest.mark.gpu
@pytest.mark.parametrize("Hq,Hkv,lens,part", [(8, 2, (300, 77, 515, 1, 64), 0), (4, 4, (130, 700), 64),
                                              (16, 8, tuple([40] * 70), 0), (8, 1, (2500,), 0),
                                              (14, 2, (300, 77, 33), 0)])
def test_fp8_pool_write_offload_reload_decode(Hq, Hkv, lens, part):
    """8-bit pool end to end: the codes lkv_write_kv stores equal the oracle's bit for bit, an offload image is
    those bytes (half the bf16 size), and decode attention over the codes matches the oracle within the bf16
    tolerance - unsplit, split into 64-token partitions, with the library's own split of a small batch, and with
    two-wavefront workgroups (70 x 8 kv heads)."""
    from paper_2410_00428_amd import binding as lkv, workloads as wl
    from tests import gpu_harness as H
    k_scale, v_scale = 0.037, 0.0125
    kw = dict(decode_partition=part) if part else {}
    shape, c, o, pool = _fp8_pair(Hq, Hkv, lens, k_scale, v_scale, 41, **kw)
    bf = wl.KVShape(1, Hq, Hkv, 128, 16, "bf16")
    B, T = len(lens), sum(lens)
    slots = []
    for s, n in enumerate(lens):
        c.alloc_layer_blocks(s, 0, n + 1)
        o.alloc_layer_blocks(s, 0, n + 1)
        slots.append(c.build_slot_mapping(s, 0, 0, n))
        assert np.array_equal(slots[-1], o.slot_mapping(s, 0, 0, n))
    slots = np.concatenate(slots)
    _, K, V = wl.qkv(41, 0, T, bf, 1.0)
    c.write_kv(0, H.to_dev(K), H.to_dev(V), H.to_dev(slots), T)
    o.write_kv(K, V, slots)
    torch.cuda.synchronize()
    assert H.pool_as_oracle_view(pool, o).tobytes() == o.pool.tobytes(), "codes differ"
    assert c.block_bytes == 16 * 2 * Hkv * 128
    # offload image of sequence 0 and reload into the same blocks after wiping them
    ids = c.get_block_table(0, 0)
    buf = H.pinned_bytes(len(ids) * c.block_bytes)
    c.pack_layer_blocks(0, ids, buf)
    c.event_synchronize(0, lkv.LKV_EV_OFFLOADED)
    assert buf.numpy()[:len(ids) * c.block_bytes].tobytes() == o.pack_layer_blocks(ids).tobytes()
    pool.view(-1, c.block_bytes)[torch.from_numpy(ids.astype(np.int64)).to(H.DEV)] = 0x7F   # NaN codes everywhere
    c.unpack_layer_blocks(0, ids, buf)
    # one decode step: a new token per sequence, then attention over n + 1 positions
    q, k1, v1 = wl.decode_qkv(41, 0, 0, B, bf, 1.0)
    s1 = np.concatenate([c.build_slot_mapping(s, 0, n, 1) for s, n in enumerate(lens)])
    c.write_kv(0, H.to_dev(k1), H.to_dev(v1), H.to_dev(s1), B)
    o.write_kv(k1, v1, s1)
    bt = c.padded_block_table(range(B), 0)
    ctx = np.asarray([n + 1 for n in lens], dtype=np.int32)
    Od = H.empty_like_storage(q.shape, "bf16")
    Od.fill_(0x7FC0)
    c.paged_decode_attention(0, H.to_dev(q), Od, H.to_dev(bt), bt.shape[1], H.to_dev(ctx), B)
    ref = o.paged_decode_attention(q, bt, ctx, threads=8)
    torch.cuda.synchronize()
    assert H.pool_as_oracle_view(pool, o).tobytes() == o.pool.tobytes(), "codes differ after reload and append"
    H.check_attention(H.to_host(Od, "bf16"), ref, "bf16", 1.0, "fp8 decode")
    c.destroy()


@pytest.mark.gpu
def test_fp8_write_every_bf16_value_gets_the_oracles_code():
    """All 65536 bf16 bit patterns (infinities, NaNs, zeros of both signs, denormals, values past 448 included)
    through lkv_write_kv at three scales: the stored byte equals the oracle's code."""
    from paper_2410_00428_amd import workloads as wl
    from tests import gpu_harness as H
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16).reshape(256, 2, 128)   # 256 tokens, 2 heads
    for k_scale, v_scale in ((1.0, 0.5), (0.037, 3.0), (1e-3, 448.0)):
        shape, c, o, pool = _fp8_pair(2, 2, (256,), k_scale, v_scale, 42)
        c.alloc_layer_blocks(0, 0, 256)
        o.alloc_layer_blocks(0, 0, 256)
        slots = c.build_slot_mapping(0, 0, 0, 256)
        c.write_kv(0, H.to_dev(allbits), H.to_dev(allbits), H.to_dev(slots), 256)
        o.write_kv(allbits, allbits, slots)
        torch.cuda.synchronize()
        got, want = H.pool_as_oracle_view(pool, o), o.pool
        bad = np.argwhere(got != want)
        assert len(bad) == 0, f"scales {k_scale}, {v_scale}: first differing element {bad[0]}: {got[tuple(bad[0])]:#x} vs {want[tuple(bad[0])]:#x}"
        c.destroy()
