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
        self.host_images: Dict[int, torch.Tensor] = {}   # layer -> pinned image (all sequences)
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
        """timing: False = no events from here; "side" = only around the side-stream transfers (their spans cannot
        be had otherwise); True = around every call (each pair of events also delays the launch it brackets)."""
        if not self.timing or (self.timing == "side" and stream is self.main):
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

    def map_prefill_layer(self, layer: int) -> np.ndarray:
        """S0 for one layer: allocate every prompt's blocks and return the slot of every token."""
        c = self.ctx
        slots = []
        for s, n in enumerate(self.lens):
            c.alloc_layer_blocks(s, layer, n)
            slots.append(c.build_slot_mapping(s, layer, 0, n))
        return np.concatenate(slots)

    def launch_prefill_layer(self, layer: int, Q, K, V, O, slots_dev, offload_to: Optional[torch.Tensor] = None,
                             attention: bool = True) -> None:
        """S1 write, S2 attention, then (if asked) S3 offload on the side stream."""
        c = self.ctx
        self._timed("write_kv", self.main, lambda: c.write_kv(layer, K, V, slots_dev, self.T, self.main))
        if attention:
            self._timed("prefill_attention", self.main,
                        lambda: c.prefill_attention(layer, Q, K, V, O, self.cu_dev, len(self.lens), max(self.lens),
                                                    self.T, True, self.main))
        if offload_to is not None:
            self.offload_layer(layer, offload_to)

    def prefill_layer(self, layer: int, Q, K, V, O, offload_to: Optional[torch.Tensor] = None,
                      attention: bool = True) -> None:
        """S0 to S3 for one layer."""
        slots_dev = torch.from_numpy(self.map_prefill_layer(layer)).to(self.device)
        self.launch_prefill_layer(layer, Q, K, V, O, slots_dev, offload_to, attention)

    def prefill_all_layers(self, Qs, Ks, Vs, O, offload: Dict[int, torch.Tensor], after_layer=None) -> None:
        """All layers of a prompt batch: the host-side mapping of every layer first (one upload), then the
        kernels of all layers back to back, each offloaded layer's copy starting behind its write.
        ``after_layer(l)``, if given, is called when layer l's launches are queued (measurement hooks)."""
        L = self.shape.num_layers
        slots = np.stack([self.map_prefill_layer(l) for l in range(L)])
        slots_dev = torch.from_numpy(slots).to(self.device)
        for l in range(L):
            i = l % len(Qs)
            self.launch_prefill_layer(l, Qs[i], Ks[i], Vs[i], O, slots_dev[l], offload.get(l))
            if after_layer is not None:
                after_layer(l)
        self._keep_prefill = slots_dev

    def layer_block_ids(self, layer: int) -> np.ndarray:
        """Block ids of every sequence's table for the layer, sequence after sequence."""
        return np.concatenate([self.ctx.get_block_table(s, layer) for s in range(len(self.lens))])

    def offload_layer(self, layer: int, buf: torch.Tensor) -> None:
        """Pack the layer's blocks of all sequences (one call, one image) and send them to pinned
        memory on the d2h stream."""
        ids = self.layer_block_ids(layer)
        self._timed("offload", self.d2h, lambda: self.ctx.pack_layer_blocks(layer, ids, buf, self.d2h))
        self.host_images[layer] = buf

    def offload_layer_pageable(self, layer: int, buf: np.ndarray) -> None:
        """The same image into ordinary host memory (Section 4: pinned memory is only a small ring that CPU
        threads of the library drain); complete once ``ctx.host_tier_synchronize(layer)`` has returned."""
        ids = self.layer_block_ids(layer)
        self._timed("offload", self.d2h, lambda: self.ctx.offload_layer_pageable(layer, ids, buf, self.d2h))
        self.host_images[layer] = buf

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
        """Give every sequence fresh blocks for the layer and bring its image back on the h2d stream."""
        c = self.ctx
        lens = lens or self.lens
        buf = self.host_images[layer]
        for s, n in enumerate(lens):
            c.alloc_layer_blocks(s, layer, n)
        ids = self.layer_block_ids(layer)
        if isinstance(buf, np.ndarray):   # pageable image: the library waits for its own CPU copies
            self._timed("reload", self.h2d, lambda: c.reload_layer_pageable(layer, ids, buf, self.h2d))
            return
        c.stream_wait_event(layer, lkv.LKV_EV_OFFLOADED, self.h2d)   # the image must be complete on the host
        self._timed("reload", self.h2d, lambda: c.unpack_layer_blocks(layer, ids, buf, self.h2d))

    def map_decode_layer(self, layer: int, step: int):
        """S0 of a decode step for one layer: one more slot per sequence, the layer's padded table."""
        c = self.ctx
        B = len(self.lens)
        slots = np.empty(B, dtype=np.int64)
        for s, n in enumerate(self.lens):
            c.alloc_layer_blocks(s, layer, n + step + 1)
            slots[s] = c.build_slot_mapping(s, layer, n + step, 1)[0]
        width = max(blocks_for(n + step + 1, self.shape.block_size) for n in self.lens)
        return slots, c.padded_block_table(range(B), layer, width)

    def decode_layer(self, layer: int, q, k, v, O, step: int = 0) -> None:
        """Append one token per sequence to the layer and attend over context n+step+1."""
        c = self.ctx
        B = len(self.lens)
        slots, bt = self.map_decode_layer(layer, step)
        ctx_lens = np.asarray([n + step + 1 for n in self.lens], dtype=np.int32)
        slots_dev = torch.from_numpy(slots).to(self.device)
        bt_dev = torch.from_numpy(bt).to(self.device)
        cl_dev = torch.from_numpy(ctx_lens).to(self.device)
        self._timed("write_kv_decode", self.main, lambda: c.write_kv(layer, k, v, slots_dev, B, self.main))
        self._timed("decode_attention", self.main,
                    lambda: c.paged_decode_attention(layer, q, O, bt_dev, bt.shape[1], cl_dev, B, self.main))
        self._keep = (slots_dev, bt_dev, cl_dev)

    def decode_all_layers(self, qs, ks, vs, O, step: int = 0) -> None:
        """One decode step over all layers: every layer's mapping first (one upload of all tables), then
        write + attention of all layers back to back."""
        c = self.ctx
        L, B = self.shape.num_layers, len(self.lens)
        maps = [self.map_decode_layer(l, step) for l in range(L)]
        slots_dev = torch.from_numpy(np.stack([m[0] for m in maps])).to(self.device)
        bt_dev = torch.from_numpy(np.stack([m[1] for m in maps])).to(self.device)
        width = bt_dev.shape[2]
        cl_dev = torch.from_numpy(np.asarray([n + step + 1 for n in self.lens], dtype=np.int32)).to(self.device)
        for l in range(L):
            self._timed("write_kv_decode", self.main, lambda: c.write_kv(l, ks[l], vs[l], slots_dev[l], B, self.main))
            self._timed("decode_attention", self.main,
                        lambda: c.paged_decode_attention(l, qs[l], O, bt_dev[l], width, cl_dev, B, self.main))
        self._keep = (slots_dev, bt_dev, cl_dev)

    def close(self) -> None:
        torch.cuda.synchronize(self.device)
        self.ctx.destroy()
