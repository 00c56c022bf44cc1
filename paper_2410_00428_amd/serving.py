"""One mixed serving iteration of the layer-wise KV cache (Section 4: in decode the host-resident layers come
back layer by layer while compute runs; in prefill a layer's new KV leaves right after it exists), with the
offloaded KV in ORDINARY host memory behind the library's small pinned ring.

A batch of decoding sequences whose context is cached, some layers on the GPU and the others on the host
(Section 3.2.2: a request keeps x layers, spread evenly), plus a few new prompts that prefill in the same
iteration.  Per layer: paged decode attention (waits for the layer's reload), write + causal attention of the
new prompts, offload of the new prompts' blocks if the layer is a host layer.  Host layers of the decode batch
pass through a ring of ``ring_layers`` sets of blocks: a layer's blocks go back to the free list as soon as its
decode attention is queued, and the reload of the host layer ``ring_layers`` places ahead takes them.

Orchestration only: every step is one call of the C ABI (``binding.LKV``); torch owns memory and streams.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Sequence, Tuple

import numpy as np
import torch

from . import binding as lkv
from .workloads import KVShape, blocks_for, cu_seqlens


class MixedIteration:
    def __init__(self, shape: KVShape, decode_lens: Sequence[int], prompt_lens: Sequence[int],
                 host_layers: Sequence[int], pool_blocks: int, ring_layers: int = 3, free_order=None,
                 device: str = "cuda:0", tier_unit_bytes: int = 0, tier_units: int = 8, tier_threads: int = 0,
                 **lkv_kw):
        self.shape, self.device = shape, torch.device(device)
        torch.cuda.set_device(self.device)
        self.dlens, self.plens = list(decode_lens), list(prompt_lens)
        self.B, self.P = len(self.dlens), len(self.plens)
        self.host_layers = sorted(host_layers)
        self.ring_layers = max(1, ring_layers)
        self.ctx = lkv.LKV(shape.num_layers, shape.num_q_heads, shape.num_kv_heads, shape.head_dim,
                           shape.block_size, pool_blocks, shape.dtype, **lkv_kw)
        if free_order is not None:
            self.ctx.pool_reset(free_order)
        self.ctx.host_tier_config(tier_unit_bytes, tier_units, tier_threads)
        self.main = torch.cuda.current_stream(self.device)
        self.d2h = torch.cuda.Stream(self.device)   # default priority
        self.h2d = torch.cuda.Stream(self.device)
        bs = shape.block_size
        self.decode_blocks = sum(blocks_for(n, bs) for n in self.dlens)
        self.prompt_blocks = sum(blocks_for(n, bs) for n in self.plens)
        self.width = max(blocks_for(n, bs) for n in self.dlens)
        self.images: Dict[int, np.ndarray] = {}          # host layer -> image of the decode batch's blocks
        self.prompt_images: Dict[int, np.ndarray] = {}   # host layer -> image of the new prompts' blocks
        self.cl_dev = torch.tensor(self.dlens, dtype=torch.int32, device=self.device)
        self.cu_dev = torch.from_numpy(cu_seqlens(self.plens)).to(self.device)
        self.T = sum(self.plens)
        self._keep: List[object] = []

    # ------------------------------------------------------------------ helpers
    def decode_ids(self, layer: int) -> np.ndarray:
        return np.concatenate([self.ctx.get_block_table(s, layer) for s in range(self.B)])

    def prompt_ids(self, layer: int) -> np.ndarray:
        return np.concatenate([self.ctx.get_block_table(self.B + i, layer) for i in range(self.P)])

    def _alloc_decode(self, layer: int) -> None:
        for s, n in enumerate(self.dlens):
            self.ctx.alloc_layer_blocks(s, layer, n)

    def _free_decode(self, layer: int) -> None:
        for s in range(self.B):
            self.ctx.free_layer_blocks(s, layer, True)

    # ------------------------------------------------------------------ the state an iteration starts from
    def decode_layer(self, layer: int, q: torch.Tensor, O: torch.Tensor) -> torch.Tensor:
        """Paged decode attention of the whole decode batch over the layer's current tables."""
        bt_dev = torch.from_numpy(self.ctx.padded_block_table(range(self.B), layer, self.width)).to(self.device)
        self.ctx.paged_decode_attention(layer, q, O, bt_dev, self.width, self.cl_dev, self.B, self.main)
        return bt_dev

    def build_cached_state(self, kv_of_layer: Callable[[int], Tuple[torch.Tensor, torch.Tensor]],
                           while_resident: Callable[[int], None] = lambda l: None,
                           progress: Callable[[str], None] = lambda s: None) -> None:
        """Every decoding sequence's context into the cache: layer by layer allocate, write K/V
        (``kv_of_layer(l)`` = device tensors [sum(decode_lens)][Hkv][d]) and, for a host layer, offload the
        layer's blocks into ordinary host memory and give the blocks back.  ``while_resident(l)`` runs after the
        write, while the layer's blocks are still on the GPU."""
        c = self.ctx
        Td = sum(self.dlens)
        for l in range(self.shape.num_layers):
            self._alloc_decode(l)
            slots = np.concatenate([c.build_slot_mapping(s, l, 0, n) for s, n in enumerate(self.dlens)])
            slots_dev = torch.from_numpy(slots).to(self.device)
            K, V = kv_of_layer(l)
            c.write_kv(l, K, V, slots_dev, Td, self.main)
            while_resident(l)
            if l in self.host_layers:
                img = self.images.get(l)
                if img is None:
                    img = self.images[l] = np.empty(self.decode_blocks * self.shape.block_bytes, dtype=np.uint8)
                c.offload_layer_pageable(l, self.decode_ids(l), img, self.d2h)   # waits for the write itself
                c.stream_wait_event(l, lkv.LKV_EV_PACKED, self.main)            # the blocks are reused below
                c.stream_wait_event(l, lkv.LKV_EV_PACKED, self.h2d)
                self._free_decode(l)
            self.main.synchronize()                                              # slots_dev, K, V may go
            progress(f"cached layer {l}" + (" -> host" if l in self.host_layers else ""))
        c.host_tier_synchronize(-1)
        for l in self.host_layers:
            if l not in self.prompt_images:
                self.prompt_images[l] = np.empty(self.prompt_blocks * self.shape.block_bytes, dtype=np.uint8)

    # ------------------------------------------------------------------ one iteration
    def _start_reload(self, layer: int) -> None:
        self._alloc_decode(layer)
        self.ctx.reload_layer_pageable(layer, self.decode_ids(layer), self.images[layer], self.h2d)

    def run(self, q_dec: Sequence[torch.Tensor], O_dec: torch.Tensor,
            prompt_qkv: Callable[[int], Tuple[torch.Tensor, torch.Tensor, torch.Tensor]], O_pf: torch.Tensor) -> None:
        """q_dec[l]: [B][Hq][d]; O_dec: [L][B][Hq][d]; prompt_qkv(l): the new prompts' packed Q, K, V of layer l;
        O_pf: [T][Hq][d] (overwritten by every layer) or one such tensor per layer.  Returns with everything queued; the caller synchronises."""
        c, L, B = self.ctx, self.shape.num_layers, self.B
        host = self.host_layers
        nxt = 0
        for _ in range(min(self.ring_layers, len(host))):   # the first host layers start coming back at once
            self._start_reload(host[nxt])
            nxt += 1
        keep: List[object] = []
        for l in range(L):
            bt_dev = self.decode_layer(l, q_dec[l], O_dec[l])
            # the new prompts of this iteration
            slots = []
            for i, n in enumerate(self.plens):
                c.alloc_layer_blocks(B + i, l, n)
                slots.append(c.build_slot_mapping(B + i, l, 0, n))
            slots_dev = torch.from_numpy(np.concatenate(slots)).to(self.device)
            Q, K, V = prompt_qkv(l)
            c.write_kv(l, K, V, slots_dev, self.T, self.main)
            Op = O_pf[l] if isinstance(O_pf, (list, tuple)) else O_pf
            c.prefill_attention(l, Q, K, V, Op, self.cu_dev, self.P, max(self.plens), self.T, True, self.main)
            keep += [bt_dev, slots_dev, Q, K, V]
            if l in host:
                c.offload_layer_pageable(l, self.prompt_ids(l), self.prompt_images[l], self.d2h)
                # this layer's set of blocks goes to the host layer ring_layers places ahead, whose scatter
                # must not start before the decode attention above has read them
                done = torch.cuda.Event()
                done.record(self.main)
                self.h2d.wait_event(done)
                self._free_decode(l)
                if nxt < len(host):
                    self._start_reload(host[nxt])
                    nxt += 1
        # the new prompts' blocks of the host layers are given back once their gathers are done
        for l in host:
            c.stream_wait_event(l, lkv.LKV_EV_PACKED, self.main)
            c.stream_wait_event(l, lkv.LKV_EV_PACKED, self.h2d)
            for i in range(self.P):
                c.free_layer_blocks(B + i, l, True)
        self._keep = keep

    def finish(self) -> None:
        """Waits for the iteration (device work and the CPU copies of the offloads)."""
        torch.cuda.synchronize(self.device)
        self.ctx.host_tier_synchronize(-1)
        self._keep = []

    def drop_prompts(self) -> None:
        """Forgets the new prompts (their retained layers' blocks go back), so that run() can be called again."""
        for i in range(self.P):
            self.ctx.free_seq(self.B + i)

    def close(self) -> None:
        self.finish()
        self.ctx.destroy()
