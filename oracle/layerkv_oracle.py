"""Plain CPU oracle of the layer-wise paged KV cache -- TEST INFRASTRUCTURE, not the product.

Written from the paper's statement of the method, not from the HIP library:

* one physical store for all layers, carved into blocks that each hold ``block_size``
  tokens of ONE layer of ONE request (Section 4: a single tensor allocated at start-up
  instead of one per layer; Section 3.2.1: blocks are allocated layer by layer);
* a block table per (request, layer) plus where that layer currently lives, GPU or host
  (Section 3.2.2: the block table is extended with per-layer location information because
  block locations differ between layers);
* offload = the bytes of a layer's blocks leave the store for host memory, reload = they
  come back, possibly into other blocks (Sections 3.2.1 and 4); neither may change a bit;
* which layers stay on the GPU when ``x`` of ``L`` are retained: spread evenly, as in the
  eight-layer example of Section 3.2.2 (keep 1,3,5,7; offload 0,2,4,6);
* attention itself is ordinary softmax attention (Section 2.1.1), done in ``attention.c``.

Readings taken where the paper is silent (block size, free-list discipline, the in-block
element order, what a decode step appends) are listed in the repository's design notes;
this file implements them in the most literal way available: Python lists and NumPy
indexing, no blocking, no fusion.

parity unpinned: nothing here concerns speed or the paper's latency figures.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

GPU, HOST = "gpu", "host"


class NoBlocks(RuntimeError):
    """The free list cannot cover an allocation (the request would have to queue, Section 2.2)."""


class NotResident(RuntimeError):
    """The layer's blocks are not in the GPU pool (offloaded, or never allocated)."""


def retained_layers(num_layers: int, x: int) -> List[int]:
    """Indices of the ``x`` layers kept on the GPU, spread evenly over ``num_layers``.

    Layer ``l`` is kept when the running quota ``floor((l+1)*x/L)`` steps up at ``l``;
    for L=8, x=4 this gives 1,3,5,7, the example of Section 3.2.2.
    """
    if not 0 <= x <= num_layers:
        raise ValueError("x out of range")
    return [l for l in range(num_layers) if ((l + 1) * x) // num_layers > (l * x) // num_layers]


class LayerKVOracle:
    """Block pool, per-layer tables and residency; byte-exact write / pack / unpack."""

    def __init__(self, num_layers: int, num_q_heads: int, num_kv_heads: int, head_dim: int,
                 block_size: int, num_pool_blocks: int, dtype: str, k_scale: float = 1.0, v_scale: float = 1.0):
        # "fp8": the pool holds E4M3 codes (oracle/fp8_codec.py) of K / k_scale and V / v_scale; queries, the new
        # keys and values handed to write_kv, and the outputs are bf16
        assert dtype in ("f32", "bf16", "fp8")
        assert num_q_heads % num_kv_heads == 0
        self.L, self.Hq, self.Hkv, self.d, self.bs = num_layers, num_q_heads, num_kv_heads, head_dim, block_size
        self.num_pool_blocks = num_pool_blocks
        self.dtype = dtype
        self.np_dtype = {"f32": np.float32, "bf16": np.uint16, "fp8": np.uint8}[dtype]
        self.in_dtype = np.float32 if dtype == "f32" else np.uint16       # what write_kv is given
        self.k_scale, self.v_scale = float(k_scale), float(v_scale)
        # documented in-block order: [kv head][K then V][token in block][channel]
        self.pool = np.zeros((num_pool_blocks, num_kv_heads, 2, block_size, head_dim), dtype=self.np_dtype)
        self.free: List[int] = []          # a stack; the LAST element is handed out next
        self.tables: Dict[Tuple[int, int], List[int]] = {}
        self.residency: Dict[Tuple[int, int], str] = {}
        self.pool_reset(np.arange(num_pool_blocks))

    # ------------------------------------------------------------------ allocator (Section 3.2.1)
    def pool_reset(self, free_order: Sequence[int]) -> None:
        """All blocks free, no tables; ``free_order[0]`` is handed out first."""
        order = [int(b) for b in free_order]
        if sorted(order) != list(range(self.num_pool_blocks)):
            raise ValueError("free_order must be a permutation of all block ids")
        self.free = order[::-1]
        self.tables.clear()
        self.residency.clear()

    def num_free_blocks(self) -> int:
        return len(self.free)

    def alloc_layer_blocks(self, seq: int, layer: int, num_tokens_total: int) -> None:
        """Grow the table of (seq, layer) so that it covers ``num_tokens_total`` tokens."""
        if not 0 <= layer < self.L or num_tokens_total < 0:
            raise ValueError("bad layer or token count")
        # a layer that sits on the host gets fresh blocks here: that is the reload's allocation
        table = self.tables.get((seq, layer), [])
        want = -(-num_tokens_total // self.bs)
        grow = want - len(table)
        if grow > len(self.free):
            raise NoBlocks(f"need {grow} blocks, {len(self.free)} free")
        table = list(table)
        for _ in range(max(0, grow)):
            table.append(self.free.pop())
        self.tables[(seq, layer)] = table
        self.residency[(seq, layer)] = GPU

    def free_layer_blocks(self, seq: int, layer: int, to_host: bool = False) -> None:
        """Give the blocks of (seq, layer) back, in table order (so the last one is reused first)."""
        table = self.tables.pop((seq, layer))
        self.free.extend(table)
        if to_host:
            self.residency[(seq, layer)] = HOST
        else:
            self.residency.pop((seq, layer), None)

    def free_seq(self, seq: int) -> None:
        """A finished request releases every layer it holds, lowest layer first (Section 2.2)."""
        for layer in range(self.L):
            if (seq, layer) in self.tables:
                self.free_layer_blocks(seq, layer)
            self.residency.pop((seq, layer), None)

    def block_table(self, seq: int, layer: int) -> List[int]:
        return list(self.tables.get((seq, layer), []))

    def layer_residency(self, seq: int, layer: int) -> Optional[str]:
        return self.residency.get((seq, layer))

    def slot_mapping(self, seq: int, layer: int, pos0: int, count: int) -> np.ndarray:
        """Slot of token position p: ``table[p // bs] * bs + p % bs`` (paging, Section 2.1.2)."""
        if self.residency.get((seq, layer)) != GPU:
            raise NotResident(f"(seq {seq}, layer {layer}) is not in the pool")
        table = self.tables[(seq, layer)]
        out = np.empty(count, dtype=np.int64)
        for i in range(count):
            p = pos0 + i
            out[i] = table[p // self.bs] * self.bs + p % self.bs
        return out

    def padded_block_table(self, seqs: Sequence[int], layer: int, width: Optional[int] = None) -> np.ndarray:
        tabs = [self.tables[(s, layer)] for s in seqs]
        width = width or max(len(t) for t in tabs)
        out = np.full((len(seqs), width), -1, dtype=np.int32)
        for i, t in enumerate(tabs):
            out[i, :len(t)] = t
        return out

    # ------------------------------------------------------------------ data movement
    def write_kv(self, K: np.ndarray, V: np.ndarray, slot_mapping: np.ndarray) -> None:
        """Token t's keys and values (all KV heads) go to slot ``slot_mapping[t]``; negative = skip."""
        assert K.shape == V.shape and K.shape[1:] == (self.Hkv, self.d) and K.dtype == self.in_dtype
        if self.dtype == "fp8":
            from oracle import fp8_codec
            K, V = fp8_codec.quantize_bf16_bits(K, self.k_scale), fp8_codec.quantize_bf16_bits(V, self.v_scale)
        for t in range(K.shape[0]):
            slot = int(slot_mapping[t])
            if slot < 0:
                continue
            b, off = divmod(slot, self.bs)
            self.pool[b, :, 0, off, :] = K[t]
            self.pool[b, :, 1, off, :] = V[t]

    def pack_layer_blocks(self, block_ids: Sequence[int]) -> np.ndarray:
        """Offload image: block ``block_ids[i]`` verbatim at byte offset ``i * block_bytes``."""
        out = np.empty((len(block_ids),) + self.pool.shape[1:], dtype=self.np_dtype)
        for i, b in enumerate(block_ids):
            out[i] = self.pool[int(b)]
        return out.reshape(-1).view(np.uint8)

    def unpack_layer_blocks(self, block_ids: Sequence[int], image: np.ndarray) -> None:
        """Reload: chunk i of the image becomes block ``block_ids[i]`` (ids may differ from pack's)."""
        chunks = np.ascontiguousarray(image).view(self.np_dtype).reshape((len(block_ids),) + self.pool.shape[1:])
        for i, b in enumerate(block_ids):
            self.pool[int(b)] = chunks[i]

    def gather_layer_kv(self, seq: int, layer: int, n: int) -> Tuple[np.ndarray, np.ndarray]:
        """Keys and values of positions 0..n-1 read back through the table: [n][Hkv][d] each."""
        K = np.empty((n, self.Hkv, self.d), dtype=self.np_dtype)
        V = np.empty_like(K)
        table = self.tables[(seq, layer)]
        for p in range(n):
            b, off = table[p // self.bs], p % self.bs
            K[p] = self.pool[b, :, 0, off, :]
            V[p] = self.pool[b, :, 1, off, :]
        return K, V

    # ------------------------------------------------------------------ attention (C)
    def prefill_attention(self, Q, K, V, cu_seqlens, causal=True, scale=None, acc="f64", threads=1):
        # prompts are attended in the precision they arrive in; the pool's format plays no part
        return prefill_attention(Q, K, V, cu_seqlens, "bf16" if self.dtype == "fp8" else self.dtype, causal, scale,
                                 acc, threads)

    def paged_decode_attention(self, Q, block_table, context_lens, scale=None, acc="f64", threads=1):
        if self.dtype == "fp8":
            # the stored values are code * scale: the codes' exact values go through the float32 path of the same
            # routine, k_scale joins the softmax scale and v_scale multiplies the result
            from oracle import fp8_codec
            q32 = (np.ascontiguousarray(Q, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
            sm = (float(self.d) ** -0.5 if scale is None else float(scale)) * self.k_scale
            return paged_decode_attention(q32, fp8_codec.decode(self.pool), block_table, context_lens, self.bs, "f32",
                                          sm, acc, threads) * self.v_scale
        return paged_decode_attention(Q, self.pool, block_table, context_lens, self.bs, self.dtype,
                                      scale, acc, threads)


# ---------------------------------------------------------------------- ctypes access to attention.c
_lib = None


def _clib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build.build())
        i32, i64, dbl, ptr = ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        for sfx in ("f64", "f32"):
            f = getattr(_lib, f"orc_prefill_attention_{sfx}")
            f.argtypes = [ptr, ptr, ptr, ptr, ptr, i32, i32, i32, i32, dbl, i32, i32, i32]
            f.restype = i32
            f = getattr(_lib, f"orc_prefill_attention_rows_{sfx}")
            f.argtypes = [ptr, ptr, ptr, ptr, ptr, i32, i32, i32, i32, dbl, i32, i32, ptr, ptr, i64, i32]
            f.restype = i32
            f = getattr(_lib, f"orc_paged_decode_attention_{sfx}")
            f.argtypes = [ptr, ptr, ptr, ptr, i32, ptr, i32, i32, i32, i32, i32, i64, dbl, i32, i32]
            f.restype = i32
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(a: np.ndarray, dtype: str) -> np.ndarray:
    want = np.float32 if dtype == "f32" else np.uint16
    if a.dtype != want:
        raise TypeError(f"expected {want} storage for dtype {dtype}, got {a.dtype}")
    return np.ascontiguousarray(a)


def prefill_attention(Q, K, V, cu_seqlens, dtype: str, causal=True, scale=None, acc="f64", threads=1):
    """Causal (or full) softmax attention on packed sequences; returns float64 [T][Hq][d]."""
    Q, K, V = _check(Q, dtype), _check(K, dtype), _check(V, dtype)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    T, Hq, d = Q.shape
    Hkv = K.shape[1]
    assert K.shape == V.shape == (T, Hkv, d) and cu[-1] == T
    scale = float(d) ** -0.5 if scale is None else float(scale)
    O = np.zeros((T, Hq, d), dtype=np.float64)
    rc = getattr(_clib(), f"orc_prefill_attention_{acc}")(
        _p(Q), _p(K), _p(V), _p(O), _p(cu), len(cu) - 1, Hq, Hkv, d, scale, int(bool(causal)),
        0 if dtype == "f32" else 1, threads)
    if rc:
        raise ValueError("orc_prefill_attention: bad arguments")
    return O


def prefill_attention_rows(Q, K, V, cu_seqlens, dtype: str, tok, head, causal=True, scale=None,
                           acc="f64", threads=1):
    """Sampled output rows (global token index, q head) of the same attention; float64 [n][d]."""
    Q, K, V = _check(Q, dtype), _check(K, dtype), _check(V, dtype)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    tok = np.ascontiguousarray(tok, dtype=np.int64)
    head = np.ascontiguousarray(head, dtype=np.int32)
    T, Hq, d = Q.shape
    Hkv = K.shape[1]
    scale = float(d) ** -0.5 if scale is None else float(scale)
    O = np.zeros((len(tok), d), dtype=np.float64)
    rc = getattr(_clib(), f"orc_prefill_attention_rows_{acc}")(
        _p(Q), _p(K), _p(V), _p(O), _p(cu), len(cu) - 1, Hq, Hkv, d, scale, int(bool(causal)),
        0 if dtype == "f32" else 1, _p(tok), _p(head), len(tok), threads)
    if rc:
        raise ValueError("orc_prefill_attention_rows: bad arguments")
    return O


def paged_decode_attention(Q, pool, block_table, context_lens, block_size: int, dtype: str,
                           scale=None, acc="f64", threads=1):
    """One query token per sequence over keys/values fetched through ``block_table``; float64 [B][Hq][d]."""
    Q = _check(Q, dtype)
    pool = _check(pool, dtype)
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    cl = np.ascontiguousarray(context_lens, dtype=np.int32)
    B, Hq, d = Q.shape
    nblk, Hkv, two, bs, d2 = pool.shape
    assert two == 2 and bs == block_size and d2 == d and bt.shape[0] == B == cl.shape[0]
    scale = float(d) ** -0.5 if scale is None else float(scale)
    O = np.zeros((B, Hq, d), dtype=np.float64)
    rc = getattr(_clib(), f"orc_paged_decode_attention_{acc}")(
        _p(Q), _p(pool), _p(O), _p(bt), bt.shape[1], _p(cl), B, Hq, Hkv, d, bs, nblk, scale,
        0 if dtype == "f32" else 1, threads)
    if rc:
        raise ValueError("orc_paged_decode_attention: bad arguments (table entry out of range?)")
    return O
