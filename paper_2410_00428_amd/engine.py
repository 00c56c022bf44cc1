"""Per-layer driver of the hot path: the order in which the paper's execution engine issues the
steps (Section 4: in prefill a layer's offload starts right after that layer's KV exists and
overlaps later compute; in decode host-resident layers come back layer by layer).

Orchestration only: every step is one call of the C ABI (``binding.LKV``); tensors are torch
device buffers used as plain memory.  Used by ``bench.py``, the smoke check and the full-size
parity tests so that they all time and test the same launch configuration.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as lkv
from .workloads import KVShape, blocks_for, cu_seqlens


class LayerKVEngine:
    def __init__(self, shape: KVShape, pool_blocks: int, free_order: Optional[np.ndarray] = None,
                 device: str = "cuda:0", **lkv_kw):
        self.shape, self.device = shape, torch.device(device)
        torch.cuda.set_device(self.device)
        self.ctx = lkv.LKV(shape.num_layers, shape.num_q_heads, shape.num_kv_heads, shape.head_dim,
                           shape.block_size, pool_blocks, shape.dtype, **lkv_kw)
        self.free_order = free_order
        if free_order is not None:
            self.ctx.pool_reset(free_order)
        self.main = torch.cuda.current_stream(self.device)
        self.d2h = torch.cuda.Stream(self.device)   # offload stream (default priority)
        self.h2d = torch.cuda.Stream(self.device)   # reload stream
        self.lens: List[int] = []
        self.host_images: Dict[int, List[torch.Tensor]] = {}   # layer -> pinned image per sequence
        self.timers: Dict[str, list] = {}
        self.timing = False

    # ------------------------------------------------------------------ helpers
    def reset(self) -> None:
        if self.free_order is not None:
            self.ctx.pool_reset(self.free_order)
        else:
            for s in range(len(self.lens)):
                self.ctx.free_seq(s)
        self.lens = []

    def _timed(self, name: str, stream, fn):
        if not self.timing:
            return fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        fn()
        b.record(stream)
        self.timers.setdefault(name, []).append((a, b))

    def elapsed_ms(self) -> Dict[str, List[float]]:
        torch.cuda.synchronize(self.device)
        return {k: [a.elapsed_time(b) for a, b in v] for k, v in self.timers.items()}

    def pinned(self, nbytes: int) -> torch.Tensor:
        return torch.empty(max(nbytes, 1), dtype=torch.uint8, pin_memory=True)

    # ------------------------------------------------------------------ prefill (S0, S1, S2, S3)
    def begin_prompts(self, lens: Sequence[int]) -> None:
        self.lens = list(lens)
        self.cu = cu_seqlens(lens)
        self.cu_dev = torch.from_numpy(self.cu).to(self.device)
        self.T = int(self.cu[-1])

    def prefill_layer(self, layer: int, Q, K, V, O, offload_to: Optional[List[torch.Tensor]] = None,
                      attention: bool = True) -> None:
        """S0 allocate + map, S1 write, S2 attention, then (if asked) S3 offload on the side stream."""
        c = self.ctx
        slots = []
        for s, n in enumerate(self.lens):
            c.alloc_layer_blocks(s, layer, n)
            slots.append(c.build_slot_mapping(s, layer, 0, n))
        slots_dev = torch.from_numpy(np.concatenate(slots)).to(self.device, non_blocking=False)
        self._timed("write_kv", self.main, lambda: c.write_kv(layer, K, V, slots_dev, self.T, self.main))
        if attention:
            self._timed("prefill_attention", self.main,
                        lambda: c.prefill_attention(layer, Q, K, V, O, self.cu_dev, len(self.lens), max(self.lens),
                                                    self.T, True, self.main))
        if offload_to is not None:
            self.offload_layer(layer, offload_to)

    def offload_layer(self, layer: int, bufs: List[torch.Tensor]) -> None:
        """Pack every sequence's blocks of the layer and send them to pinned memory on the d2h stream."""
        c = self.ctx
        def go():
            for s in range(len(self.lens)):
                c.pack_layer_blocks(layer, c.get_block_table(s, layer), bufs[s], self.d2h)
        self._timed("offload", self.d2h, go)
        self.host_images[layer] = bufs

    def release_offloaded(self, layer: int) -> None:
        """The layer's blocks go back to the free list (host logic); the data lives on the host now.
        The main stream is ordered behind the gather so that whoever reuses the blocks writes later."""
        c = self.ctx
        c.stream_wait_event(layer, lkv.LKV_EV_PACKED, self.main)
        c.stream_wait_event(layer, lkv.LKV_EV_PACKED, self.h2d)
        for s in range(len(self.lens)):
            c.free_layer_blocks(s, layer, True)

    # ------------------------------------------------------------------ reload + decode (S4, S5)
    def reload_layer(self, layer: int, lens: Optional[Sequence[int]] = None) -> None:
        c = self.ctx
        lens = lens or self.lens
        bufs = self.host_images[layer]
        c.stream_wait_event(layer, lkv.LKV_EV_OFFLOADED, self.h2d)   # the image must be complete on the host
        def go():
            for s, n in enumerate(lens):
                c.alloc_layer_blocks(s, layer, n)
                c.unpack_layer_blocks(layer, c.get_block_table(s, layer), bufs[s], self.h2d)
        self._timed("reload", self.h2d, go)

    def decode_layer(self, layer: int, q, k, v, O, step: int = 0) -> None:
        """Append one token per sequence to the layer and attend over context n+step+1."""
        c = self.ctx
        B = len(self.lens)
        slots = np.empty(B, dtype=np.int64)
        for s, n in enumerate(self.lens):
            c.alloc_layer_blocks(s, layer, n + step + 1)
            slots[s] = c.build_slot_mapping(s, layer, n + step, 1)[0]
        bt = c.padded_block_table(range(B), layer)
        ctx_lens = np.asarray([n + step + 1 for n in self.lens], dtype=np.int32)
        slots_dev = torch.from_numpy(slots).to(self.device)
        bt_dev = torch.from_numpy(bt).to(self.device)
        cl_dev = torch.from_numpy(ctx_lens).to(self.device)
        self._timed("write_kv_decode", self.main, lambda: c.write_kv(layer, k, v, slots_dev, B, self.main))
        self._timed("decode_attention", self.main,
                    lambda: c.paged_decode_attention(layer, q, O, bt_dev, bt.shape[1], cl_dev, B, self.main))
        self._keep = (slots_dev, bt_dev, cl_dev)

    def close(self) -> None:
        torch.cuda.synchronize(self.device)
        self.ctx.destroy()
