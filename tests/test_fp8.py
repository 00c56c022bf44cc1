"""The 8-bit KV-cache format (OCP E4M3, the paper's Future Work made concrete): pins of the oracle's codec, then
the library against it."""
from fractions import Fraction as F

import numpy as np
import pytest

from oracle import fp8_codec as fp8

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
