"""Seeded synthetic inputs for the layer-wise paged KV cache path.

This module only draws random numbers and lays them out; it contains none of the
method's arithmetic (no allocator, no slot mapping, no attention).  It is the one module
that both the CPU oracle's tests and the HIP path's tests/bench feed from, so that both
sides see exactly the same bits.

The workloads stand in for the paper's evaluation traffic (Section 5.1: LLaMA-2-7B,
Yi-34B-200K and LLaMA-3.1-70B serving ShareGPT prompts and fixed-length prompts from 128
to 16k tokens): same KV shapes and length ranges, synthetic values.

RNG recipe: ``numpy.random.Generator(PCG64(child))`` where ``child`` comes from
``SeedSequence(241000 + config_number).spawn(...)`` in the fixed stream order
``lengths, free_list, q, k, v, decode, schedule``; tensors are ``standard_normal(float32)``
times a scale, then rounded once (round-to-nearest-even) to the config's dtype.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np

SEED_BASE = 241000
STREAMS = ("lengths", "free_list", "q", "k", "v", "decode", "schedule")


# --------------------------------------------------------------------------- dtype helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def elem_size(dtype: str) -> int:
    return {"f32": 4, "bf16": 2, "fp8": 1}[dtype]   # "fp8": one-byte codes in the pool, bf16 everywhere else


def storage_dtype(dtype: str):
    return {"f32": np.float32, "bf16": np.uint16, "fp8": np.uint16}[dtype]   # of the tensors handed to the calls


def to_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    return x.astype(np.float32) if dtype == "f32" else bf16_bits_to_f32(x)   # bf16 and fp8 pools: bf16 tensors


# --------------------------------------------------------------------------- shapes / configs
@dataclass(frozen=True)
class KVShape:
    num_layers: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    dtype: str  # "f32" | "bf16" | "fp8" (pool of E4M3 codes, tensors bf16)

    @property
    def token_bytes(self) -> int:  # tau: K and V of one token in one layer
        return 2 * self.num_kv_heads * self.head_dim * elem_size(self.dtype)

    @property
    def block_bytes(self) -> int:  # beta: one layer-block
        return self.block_size * self.token_bytes


@dataclass(frozen=True)
class Workload:
    number: int
    name: str
    shape: KVShape
    data_scale: float            # multiplier applied to N(0,1) draws
    prompt_lens: Tuple[int, ...]  # sequences that are prefilled
    decode_lens: Tuple[int, ...]  # sequences that only decode (context already cached)
    decode_steps: int
    offload_layers: Tuple[int, ...]
    pool_blocks: int
    note: str = ""


SHAPE_TINY = KVShape(2, 4, 4, 64, 16, "f32")
SHAPE_7B = KVShape(32, 32, 32, 128, 16, "bf16")
SHAPE_70B = KVShape(80, 64, 8, 128, 16, "bf16")


# Layers sent to host memory in workloads 3 and 5 ("24 of 32", "75 %"): every layer except
# 3, 7, 11, ..., 31.  Written out as data; the even-spread rule of Section 3.2.2 that
# produces this set is implemented, and tested, on each side separately.
OFFLOAD_24_OF_32 = tuple(l for l in range(32) if l % 4 != 3)


def rng_for(config_number: int, stream: str, index: int = 0) -> np.random.Generator:
    """Independent child stream ``stream`` (optionally sub-indexed, e.g. per layer)."""
    pos = STREAMS.index(stream)
    # spawn_key (pos,) is the pos-th child of SeedSequence(seed); (pos, index) its index-th child
    key = (pos,) if index == 0 else (pos, index)
    child = np.random.SeedSequence(SEED_BASE + config_number, spawn_key=key)
    return np.random.Generator(np.random.PCG64(child))


def lognormal_lengths(rng: np.random.Generator, count: int, median: int, sigma: float,
                      lo: int, hi: int) -> Tuple[int, ...]:
    x = rng.lognormal(mean=float(np.log(median)), sigma=sigma, size=count)
    return tuple(int(v) for v in np.clip(np.rint(x), lo, hi).astype(np.int64))


def uniform_lengths(rng: np.random.Generator, count: int, lo: int, hi: int) -> Tuple[int, ...]:
    return tuple(int(v) for v in rng.integers(lo, hi + 1, size=count))


def blocks_for(n_tokens: int, block_size: int) -> int:
    return -(-n_tokens // block_size)


def workload(number: int, decode_seqs_cfg5: int = 64) -> Workload:
    """The five benchmark/parity workloads."""
    if number == 1:
        s = SHAPE_TINY
        return Workload(1, "tiny-fp32", s, 1.0, (128, 200, 317, 512), (), 1, (1,),
                        pool_blocks=s.num_layers * 128,
                        note="pool read as 128 block ids per layer (256 layer-blocks)")
    if number == 2:
        s = SHAPE_7B
        lens = (2048,) * 8
        per_layer = sum(blocks_for(n + 1, s.block_size) for n in lens)
        return Workload(2, "llama2-7b-8x2048", s, 128 ** -0.5, lens, (), 1,
                        tuple(range(16, 32)), pool_blocks=per_layer * s.num_layers)
    if number == 3:
        s = SHAPE_7B
        lens = (16384,) * 4
        per_layer = sum(blocks_for(n + 64, s.block_size) for n in lens)
        return Workload(3, "llama2-7b-4x16384", s, 128 ** -0.5, lens, (), 64,
                        OFFLOAD_24_OF_32, pool_blocks=per_layer * s.num_layers)
    if number == 4:
        s = SHAPE_70B
        lens = lognormal_lengths(rng_for(4, "lengths"), 16, 4096, 1.0, 128, 16384)
        per_layer = sum(blocks_for(n, s.block_size) for n in lens)
        # the pool holds every layer plus head-room for the dummy sequences that fragment it
        return Workload(4, "llama2-70b-gqa-decode", s, 128 ** -0.5, (), lens, 1, (),
                        pool_blocks=int(per_layer * s.num_layers * 1.25) + 1024)
    if number == 5:
        s = SHAPE_7B
        lens = uniform_lengths(rng_for(5, "lengths"), decode_seqs_cfg5, 128, 16384)
        per_layer = sum(blocks_for(n + 1, s.block_size) for n in lens) + 2 * blocks_for(8192, s.block_size)
        return Workload(5, "llama2-7b-mixed", s, 1.0, (8192, 8192), lens, 1,
                        OFFLOAD_24_OF_32, pool_blocks=per_layer * s.num_layers)
    raise ValueError(f"no workload {number}")


# --------------------------------------------------------------------------- tensors
def normal_tensor(rng: np.random.Generator, shape: Sequence[int], scale: float, dtype: str) -> np.ndarray:
    """N(0,1)*scale drawn in float32 and rounded once to ``dtype``; f32 array or bf16 bit patterns."""
    x = rng.standard_normal(tuple(shape), dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    return x if dtype == "f32" else f32_to_bf16_bits(x)   # also for "fp8": only the pool is 8-bit


def normal_tensor_chunked(config_number: int, stream: str, index: int, shape: Sequence[int], scale: float,
                          dtype: str, rows_per_chunk: int = 4096, threads: int = 16) -> np.ndarray:
    """The same kind of tensor for sizes where one generator would take minutes (GiB-sized caches): rows
    [c * rows_per_chunk, (c + 1) * rows_per_chunk) come from the child stream (stream, index, c), so the result does
    not depend on how many threads draw the chunks."""
    from concurrent.futures import ThreadPoolExecutor
    shape = tuple(shape)
    out = np.empty(shape, dtype=np.float32 if dtype == "f32" else np.uint16)
    pos = STREAMS.index(stream)

    def draw(c: int) -> None:
        a, b = c * rows_per_chunk, min(shape[0], (c + 1) * rows_per_chunk)
        child = np.random.SeedSequence(SEED_BASE + config_number, spawn_key=(pos, index, c))
        out[a:b] = normal_tensor(np.random.Generator(np.random.PCG64(child)), (b - a,) + shape[1:], scale, dtype)

    chunks = range(-(-shape[0] // rows_per_chunk))
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(draw, chunks))
    return out


def qkv(config_number: int, layer: int, num_tokens: int, shape: KVShape, scale: float,
        q_gain: float = 1.0) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Token-major Q [T][Hq][d], K and V [T][Hkv][d] for one layer (independent streams per layer)."""
    q = normal_tensor(rng_for(config_number, "q", layer), (num_tokens, shape.num_q_heads, shape.head_dim),
                      scale * q_gain, shape.dtype)
    k = normal_tensor(rng_for(config_number, "k", layer), (num_tokens, shape.num_kv_heads, shape.head_dim),
                      scale, shape.dtype)
    v = normal_tensor(rng_for(config_number, "v", layer), (num_tokens, shape.num_kv_heads, shape.head_dim),
                      scale, shape.dtype)
    return q, k, v


def decode_qkv(config_number: int, layer: int, step: int, num_seqs: int, shape: KVShape, scale: float,
               q_gain: float = 1.0) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One new token per sequence: q [B][Hq][d], k and v [B][Hkv][d]."""
    rng = rng_for(config_number, "decode", layer * 4096 + step)
    q = normal_tensor(rng, (num_seqs, shape.num_q_heads, shape.head_dim), scale * q_gain, shape.dtype)
    k = normal_tensor(rng, (num_seqs, shape.num_kv_heads, shape.head_dim), scale, shape.dtype)
    v = normal_tensor(rng, (num_seqs, shape.num_kv_heads, shape.head_dim), scale, shape.dtype)
    return q, k, v


def free_list_order(config_number: int, pool_blocks: int, index: int = 0) -> np.ndarray:
    """Seeded permutation of the physical block ids; element 0 is handed out first."""
    return rng_for(config_number, "free_list", index).permutation(pool_blocks).astype(np.int32)


def cu_seqlens(lens: Sequence[int]) -> np.ndarray:
    out = np.zeros(len(lens) + 1, dtype=np.int32)
    out[1:] = np.cumsum(np.asarray(lens, dtype=np.int64))
    return out


# --------------------------------------------------------------------------- allocation schedules
@dataclass
class AllocOp:
    op: str          # "alloc" | "free"
    seq: int
    layer: int
    tokens: int = 0  # for alloc: new total token count of (seq, layer)


def fragmenting_schedule(config_number: int, layer: int, lens: Sequence[int], block_size: int,
                         dummy_base: int = 1 << 20) -> List[AllocOp]:
    """A list of allocator calls for one layer that leaves the real sequences' tables fragmented.

    The real sequences grow round-robin in bursts of 1-8 blocks; between bursts a dummy
    sequence takes 1-4 blocks, and every other dummy is freed a few bursts later so that
    its blocks are handed to a different real sequence.  Both the oracle's allocator and
    the library's replay the same list; the list itself contains no allocator logic.
    """
    rng = rng_for(config_number, "schedule", layer)
    ops: List[AllocOp] = []
    have = [0] * len(lens)
    need = [blocks_for(n, block_size) for n in lens]
    dummy = 0
    pending_free: List[int] = []
    while any(h < n for h, n in zip(have, need)):
        for s in range(len(lens)):
            if have[s] >= need[s]:
                continue
            burst = int(rng.integers(1, 9))
            have[s] = min(need[s], have[s] + burst)
            ops.append(AllocOp("alloc", s, layer, min(lens[s], have[s] * block_size)))
            d = dummy_base + dummy
            dummy += 1
            ops.append(AllocOp("alloc", d, layer, int(rng.integers(1, 5)) * block_size))
            pending_free.append(d)
            if len(pending_free) > 3:
                ops.append(AllocOp("free", pending_free.pop(0), layer))
    for d in pending_free:
        ops.append(AllocOp("free", d, layer))
    return ops


def sample_rows(rng: np.random.Generator, n: int, count: int, always: Sequence[int] = (0, 15, 16)) -> np.ndarray:
    """Row indices in [0, n): the fixed ones (clipped), n-1, and seeded others, sorted unique."""
    fixed = [r for r in always if r < n] + [n - 1]
    extra = rng.integers(0, n, size=max(0, count - len(fixed)))
    return np.unique(np.concatenate([np.asarray(fixed, dtype=np.int64), extra.astype(np.int64)]))
