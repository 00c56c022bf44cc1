"""ctypes binding of ``liblkv.so``: the same names as ``include/lkv.h``, argument marshalling only.

Every step of the path runs inside the library's HIP kernels; nothing here computes on KV
data and there is no fallback: if the library is missing or a call fails, an exception is
raised.  Device buffers are passed as integer addresses (``tensor.data_ptr()``), streams as
``torch.cuda.Stream.cuda_stream`` integers (0 = default stream).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liblkv.so")

LKV_OK, LKV_ERR_INVALID_ARG, LKV_ERR_NO_BLOCKS, LKV_ERR_NOT_RESIDENT = 0, 1, 2, 3
LKV_ERR_HOST_MEMORY, LKV_ERR_DEVICE, LKV_ERR_UNSUPPORTED = 4, 5, 6
LKV_F32, LKV_BF16, LKV_FP8_E4M3 = 0, 1, 2
LKV_RES_NONE, LKV_RES_GPU, LKV_RES_HOST, LKV_RES_IN_FLIGHT = 0, 1, 2, 3
LKV_EV_KV_WRITTEN, LKV_EV_PACKED, LKV_EV_OFFLOADED, LKV_EV_RELOADED = 0, 1, 2, 3
STATUS_NAMES = {0: "LKV_OK", 1: "LKV_ERR_INVALID_ARG", 2: "LKV_ERR_NO_BLOCKS", 3: "LKV_ERR_NOT_RESIDENT",
                4: "LKV_ERR_HOST_MEMORY", 5: "LKV_ERR_DEVICE", 6: "LKV_ERR_UNSUPPORTED"}

# every symbol include/lkv.h declares
EXPORTS = (
    "lkv_create", "lkv_create_logical", "lkv_destroy", "lkv_last_error", "lkv_pool_info",
    "lkv_pool_reset", "lkv_alloc_layer_blocks", "lkv_free_layer_blocks", "lkv_free_seq",
    "lkv_get_block_table", "lkv_build_slot_mapping", "lkv_layer_residency", "lkv_num_free_blocks",
    "lkv_plan_retained_layers",
    "lkv_write_kv", "lkv_prefill_attention", "lkv_pack_layer_blocks", "lkv_unpack_layer_blocks",
    "lkv_paged_decode_attention",
    "lkv_host_tier_config", "lkv_offload_layer_pageable", "lkv_reload_layer_pageable", "lkv_host_tier_synchronize",
    "lkv_set_link_gate",
    "lkv_stream_wait_event", "lkv_event_synchronize", "lkv_set_profiling", "lkv_get_stats",
    "lkv_reserve_decode_workspace", "lkv_paged_decode_attention_static",
    "lkv_prefill_time", "lkv_offload_time", "lkv_plan_offload", "lkv_allow_prefill_time", "lkv_max_prefills",
    "lkv_forecast_avail", "lkv_pressure_offload",
)


class LkvConfig(ctypes.Structure):
    _fields_ = [("num_layers", ctypes.c_int32), ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("num_pool_blocks", ctypes.c_int64), ("softmax_scale", ctypes.c_float),
                ("decode_partition", ctypes.c_int32), ("pool", ctypes.c_void_p), ("staging_bytes", ctypes.c_int64),
                ("k_scale", ctypes.c_float), ("v_scale", ctypes.c_float)]


class LkvStats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in
                ("write_kv_calls", "write_kv_bytes", "prefill_calls", "decode_calls", "pack_calls", "pack_bytes",
                 "unpack_calls", "unpack_bytes", "pack_kernel_ns", "pack_kernel_bytes", "unpack_kernel_ns",
                 "unpack_kernel_bytes", "write_kernel_ns", "write_kernel_launches", "prefill_kernel_ns",
                 "prefill_kernel_launches", "decode_kernel_ns", "decode_kernel_launches",
                 "pageable_offload_calls", "pageable_offload_bytes", "pageable_reload_calls", "pageable_reload_bytes",
                 "tier_copy_bytes", "tier_copy_ns", "ring_wait_ns", "gate_busy_answers", "write_kernel_bytes")]


LINK_BUSY_FN = ctypes.CFUNCTYPE(ctypes.c_int32, ctypes.c_void_p)


class CostModel(ctypes.Structure):
    """lkv_cost_model: the prefill-time and offload-time models of the paper (Sections 3.1, 3.2.1)."""
    _fields_ = [("alpha", ctypes.c_double), ("n_param", ctypes.c_double), ("n_hidden", ctypes.c_double),
                ("device_flops", ctypes.c_double), ("beta", ctypes.c_double), ("num_layers", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("num_heads", ctypes.c_int32), ("bytes_per_elem", ctypes.c_double),
                ("link_bytes_per_s", ctypes.c_double)]


class DecodeRequest(ctypes.Structure):
    """lkv_decode_request: a decoding request as the SLO-aware scheduler sees it (Section 3.1)."""
    _fields_ = [("t_tpot", ctypes.c_double), ("n_past", ctypes.c_int64), ("t_past", ctypes.c_double),
                ("predicted_lower_bound", ctypes.c_int64)]


class LkvError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load liblkv.so (built by ``paper_2410_00428_amd.build``); raises if it is not there."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2410_00428_amd.build` "
                                "(there is no fallback path)")
    # torch ships its own copy of the HIP runtime; importing it first makes liblkv.so resolve to
    # that same copy, so torch's streams and device pointers are valid inside the library.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(path)
    i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
    P = ctypes.POINTER
    sig = {
        "lkv_create": (i32, [P(LkvConfig), P(vp)]),
        "lkv_create_logical": (i32, [P(LkvConfig), P(vp)]),
        "lkv_destroy": (None, [vp]),
        "lkv_last_error": (ctypes.c_char_p, [vp]),
        "lkv_pool_info": (i32, [vp, P(vp), P(i64), P(i64)]),
        "lkv_pool_reset": (i32, [vp, vp, i64]),
        "lkv_alloc_layer_blocks": (i32, [vp, i64, i32, i64]),
        "lkv_free_layer_blocks": (i32, [vp, i64, i32, i32]),
        "lkv_free_seq": (i32, [vp, i64]),
        "lkv_get_block_table": (i32, [vp, i64, i32, vp, i64, P(i64)]),
        "lkv_build_slot_mapping": (i32, [vp, i64, i32, i64, i64, vp]),
        "lkv_layer_residency": (i32, [vp, i64, i32, P(i32)]),
        "lkv_num_free_blocks": (i64, [vp]),
        "lkv_plan_retained_layers": (i32, [i32, i32, vp]),
        "lkv_write_kv": (i32, [vp, i32, vp, vp, vp, i64, vp]),
        "lkv_prefill_attention": (i32, [vp, i32, vp, vp, vp, vp, vp, i32, i32, i64, i32, vp]),
        "lkv_pack_layer_blocks": (i32, [vp, i32, vp, i64, vp, vp]),
        "lkv_unpack_layer_blocks": (i32, [vp, i32, vp, i64, vp, vp]),
        "lkv_paged_decode_attention": (i32, [vp, i32, vp, vp, vp, i32, vp, i32, vp]),
        "lkv_host_tier_config": (i32, [vp, i64, i32, i32]),
        "lkv_offload_layer_pageable": (i32, [vp, i32, vp, i64, vp, vp]),
        "lkv_reload_layer_pageable": (i32, [vp, i32, vp, i64, vp, vp]),
        "lkv_host_tier_synchronize": (i32, [vp, i32]),
        "lkv_set_link_gate": (i32, [vp, LINK_BUSY_FN, vp, i64, i32]),
        "lkv_stream_wait_event": (i32, [vp, i32, i32, vp]),
        "lkv_event_synchronize": (i32, [vp, i32, i32]),
        "lkv_set_profiling": (i32, [vp, i32]),
        "lkv_get_stats": (i32, [vp, P(LkvStats), i64]),
        "lkv_reserve_decode_workspace": (i32, [vp, i32, i32]),
        "lkv_paged_decode_attention_static": (i32, [vp, i32, vp, vp, vp, i32, vp, i32, vp]),
        "lkv_prefill_time": (ctypes.c_double, [P(CostModel), i64]),
        "lkv_offload_time": (ctypes.c_double, [P(CostModel), i64, i32]),
        "lkv_plan_offload": (i32, [P(CostModel), i64, P(i32), vp]),
        "lkv_allow_prefill_time": (ctypes.c_double, [P(DecodeRequest)]),
        "lkv_max_prefills": (i32, [P(DecodeRequest), i32, P(ctypes.c_double), i32, P(i32)]),
        "lkv_forecast_avail": (i32, [i64, vp, vp, i32, i64, vp, P(i32)]),
        "lkv_pressure_offload": (i32, [i64, vp, vp, i32, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    if path == LIB_PATH:
        _lib = lib
    return lib


def _ptr(x) -> int:
    """Address of a device/pinned buffer: a torch tensor, an int, or None."""
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    raise TypeError(f"cannot take the address of {type(x)}")


def _stream(s) -> int:
    if s is None:
        return 0
    if isinstance(s, int):
        return s
    return s.cuda_stream


def plan_retained_layers(num_layers: int, x: int) -> list:
    mask = np.zeros(num_layers, dtype=np.int32)
    st = load_library().lkv_plan_retained_layers(num_layers, x, mask.ctypes.data)
    if st:
        raise LkvError(st, "lkv_plan_retained_layers: bad arguments")
    return [l for l in range(num_layers) if mask[l]]


# ---------------------------------------------------------------------- host-side policy (no context)
def prefill_time(model: CostModel, seqlen: int) -> float:
    return load_library().lkv_prefill_time(ctypes.byref(model), seqlen)


def offload_time(model: CostModel, seqlen: int, x: int) -> float:
    return load_library().lkv_offload_time(ctypes.byref(model), seqlen, x)


def plan_offload(model: CostModel, seqlen: int):
    """(x, mask): the fewest layers to retain so that the offload hides behind the prefill, and which ones."""
    x = ctypes.c_int32(0)
    mask = np.zeros(max(model.num_layers, 1), dtype=np.int32)
    st = load_library().lkv_plan_offload(ctypes.byref(model), seqlen, ctypes.byref(x), mask.ctypes.data)
    if st:
        raise LkvError(st, "lkv_plan_offload: bad arguments")
    return x.value, mask[:model.num_layers]


def allow_prefill_time(t_tpot: float, n_past: int, t_past: float, predicted_lower_bound: int) -> float:
    r = DecodeRequest(t_tpot, n_past, t_past, predicted_lower_bound)
    return load_library().lkv_allow_prefill_time(ctypes.byref(r))


def max_prefills(decoding: Sequence[dict], prefill_times: Sequence[float]) -> int:
    reqs = (DecodeRequest * max(len(decoding), 1))(*[DecodeRequest(**d) for d in decoding])
    times = (ctypes.c_double * max(len(prefill_times), 1))(*prefill_times)
    n = ctypes.c_int32(0)
    st = load_library().lkv_max_prefills(reqs, len(decoding), times, len(prefill_times), ctypes.byref(n))
    if st:
        raise LkvError(st, "lkv_max_prefills: bad arguments")
    return n.value


def forecast_avail(avail0: int, released: Sequence[int], allocated: Sequence[int], threshold: int):
    """(Avail(1..T), first stage below the threshold or -1)."""
    rel = np.ascontiguousarray(released, dtype=np.int64)
    alc = np.ascontiguousarray(allocated, dtype=np.int64)
    out = np.zeros(max(len(rel), 1), dtype=np.int64)
    first = ctypes.c_int32(0)
    st = load_library().lkv_forecast_avail(avail0, rel.ctypes.data, alc.ctypes.data, len(rel), threshold, out.ctypes.data,
                                           ctypes.byref(first))
    if st:
        raise LkvError(st, "lkv_forecast_avail: bad arguments")
    return [int(v) for v in out[:len(rel)]], first.value


def pressure_offload(deficit_blocks: int, retained: Sequence[int], blocks_per_layer: Sequence[int]) -> list:
    x = np.ascontiguousarray(retained, dtype=np.int32)
    b = np.ascontiguousarray(blocks_per_layer, dtype=np.int64)
    give = np.zeros(max(len(x), 1), dtype=np.int32)
    st = load_library().lkv_pressure_offload(deficit_blocks, x.ctypes.data, b.ctypes.data, len(x), give.ctypes.data)
    if st:
        raise LkvError(st, "lkv_pressure_offload: bad arguments")
    return [int(v) for v in give[:len(x)]]


class LKV:
    """One ``lkv_ctx``.  Method names drop the ``lkv_`` prefix; arguments follow the header."""

    def __init__(self, num_layers: int, num_q_heads: int, num_kv_heads: int, head_dim: int, block_size: int,
                 num_pool_blocks: int, dtype: str, softmax_scale: float = 0.0, decode_partition: int = 0,
                 pool=None, staging_bytes: int = 0, logical_only: bool = False, k_scale: float = 0.0,
                 v_scale: float = 0.0):
        self.lib = load_library()
        self.cfg = LkvConfig(num_layers, num_q_heads, num_kv_heads, head_dim, block_size,
                             {"f32": LKV_F32, "bf16": LKV_BF16, "fp8": LKV_FP8_E4M3}[dtype], num_pool_blocks,
                             softmax_scale, decode_partition, _ptr(pool), staging_bytes, k_scale, v_scale)
        self._pool_keepalive = pool
        self.dtype = dtype
        h = ctypes.c_void_p()
        create = self.lib.lkv_create_logical if logical_only else self.lib.lkv_create
        st = create(ctypes.byref(self.cfg), ctypes.byref(h))
        if st:
            raise LkvError(st, self.lib.lkv_last_error(None).decode())
        self.h = h
        self.elem = {"f32": 4, "bf16": 2, "fp8": 1}[dtype]   # bytes per element of the POOL
        self.token_bytes = 2 * num_kv_heads * head_dim * self.elem
        self.block_bytes = block_size * self.token_bytes

    # ------------------------------------------------------------------ plumbing
    def _check(self, st: int) -> None:
        if st:
            raise LkvError(st, self.lib.lkv_last_error(self.h).decode())

    def destroy(self) -> None:
        if getattr(self, "h", None):
            self.lib.lkv_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()

    def pool_info(self):
        p, b, bb = ctypes.c_void_p(), ctypes.c_int64(), ctypes.c_int64()
        self._check(self.lib.lkv_pool_info(self.h, ctypes.byref(p), ctypes.byref(b), ctypes.byref(bb)))
        return p.value, b.value, bb.value

    # ------------------------------------------------------------------ logical state
    def pool_reset(self, free_order: Sequence[int]) -> None:
        a = np.ascontiguousarray(free_order, dtype=np.int32)
        self._check(self.lib.lkv_pool_reset(self.h, a.ctypes.data, a.size))

    def alloc_layer_blocks(self, seq: int, layer: int, num_tokens_total: int) -> None:
        self._check(self.lib.lkv_alloc_layer_blocks(self.h, seq, layer, num_tokens_total))

    def free_layer_blocks(self, seq: int, layer: int, to_host: bool = False) -> None:
        self._check(self.lib.lkv_free_layer_blocks(self.h, seq, layer, int(to_host)))

    def free_seq(self, seq: int) -> None:
        self._check(self.lib.lkv_free_seq(self.h, seq))

    def get_block_table(self, seq: int, layer: int) -> np.ndarray:
        n = ctypes.c_int64()
        st = self.lib.lkv_get_block_table(self.h, seq, layer, None, 0, ctypes.byref(n))
        if st == LKV_ERR_NOT_RESIDENT:
            self._check(st)
        out = np.empty(n.value, dtype=np.int32)
        self._check(self.lib.lkv_get_block_table(self.h, seq, layer, out.ctypes.data, out.size, ctypes.byref(n)))
        return out

    def build_slot_mapping(self, seq: int, layer: int, pos0: int, count: int) -> np.ndarray:
        out = np.empty(count, dtype=np.int64)
        self._check(self.lib.lkv_build_slot_mapping(self.h, seq, layer, pos0, count, out.ctypes.data))
        return out

    def layer_residency(self, seq: int, layer: int) -> int:
        r = ctypes.c_int32()
        self._check(self.lib.lkv_layer_residency(self.h, seq, layer, ctypes.byref(r)))
        return r.value

    def num_free_blocks(self) -> int:
        return self.lib.lkv_num_free_blocks(self.h)

    def padded_block_table(self, seqs: Sequence[int], layer: int, width: Optional[int] = None) -> np.ndarray:
        """Host-side convenience: the tables of ``seqs`` as one int32 [len(seqs)][width] array padded with -1."""
        tabs = [self.get_block_table(s, layer) for s in seqs]
        width = width or max(len(t) for t in tabs)
        out = np.full((len(seqs), width), -1, dtype=np.int32)
        for i, t in enumerate(tabs):
            out[i, :len(t)] = t
        return out

    # ------------------------------------------------------------------ device hot path
    def write_kv(self, layer: int, K, V, slot_mapping, num_tokens: int, stream=None) -> None:
        self._check(self.lib.lkv_write_kv(self.h, layer, _ptr(K), _ptr(V), _ptr(slot_mapping), num_tokens,
                                          _stream(stream)))

    def prefill_attention(self, layer: int, Q, K, V, O, cu_seqlens, num_seqs: int, max_seqlen: int,
                          total_tokens: int, causal: bool = True, stream=None) -> None:
        self._check(self.lib.lkv_prefill_attention(self.h, layer, _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(cu_seqlens),
                                                   num_seqs, max_seqlen, total_tokens, int(bool(causal)),
                                                   _stream(stream)))

    def pack_layer_blocks(self, layer: int, block_ids, pinned_dst, stream=None) -> None:
        ids = np.ascontiguousarray(block_ids, dtype=np.int32)
        self._check(self.lib.lkv_pack_layer_blocks(self.h, layer, ids.ctypes.data, ids.size, _ptr(pinned_dst),
                                                   _stream(stream)))

    def unpack_layer_blocks(self, layer: int, block_ids, pinned_src, stream=None) -> None:
        ids = np.ascontiguousarray(block_ids, dtype=np.int32)
        self._check(self.lib.lkv_unpack_layer_blocks(self.h, layer, ids.ctypes.data, ids.size, _ptr(pinned_src),
                                                     _stream(stream)))

    # ------------------------------------------------------------------ pageable host tier
    def host_tier_config(self, unit_bytes: int = 0, num_units: int = 0, threads: int = 0) -> None:
        self._check(self.lib.lkv_host_tier_config(self.h, unit_bytes, num_units, threads))

    def offload_layer_pageable(self, layer: int, block_ids, host_dst, stream=None) -> None:
        """host_dst: ordinary host memory (numpy array, CPU tensor or address) that stays alive until
        ``host_tier_synchronize(layer)`` has returned."""
        ids = np.ascontiguousarray(block_ids, dtype=np.int32)
        self._check(self.lib.lkv_offload_layer_pageable(self.h, layer, ids.ctypes.data, ids.size, _ptr(host_dst),
                                                        _stream(stream)))

    def reload_layer_pageable(self, layer: int, block_ids, host_src, stream=None) -> None:
        ids = np.ascontiguousarray(block_ids, dtype=np.int32)
        self._check(self.lib.lkv_reload_layer_pageable(self.h, layer, ids.ctypes.data, ids.size, _ptr(host_src),
                                                       _stream(stream)))

    def host_tier_synchronize(self, layer: int = -1) -> None:
        self._check(self.lib.lkv_host_tier_synchronize(self.h, layer))

    def set_link_gate(self, busy=None, delay_us: int = 0, max_checks: int = 0) -> None:
        """busy: a callable without arguments returning True while the host link is taken, or None."""
        if busy is None:
            self._gate = None
            self._check(self.lib.lkv_set_link_gate(self.h, LINK_BUSY_FN(), None, 0, 0))
            return
        cb = LINK_BUSY_FN(lambda _user: 1 if busy() else 0)
        self._check(self.lib.lkv_set_link_gate(self.h, cb, None, delay_us, max_checks))
        self._gate = cb  # the library keeps the pointer: keep the thunk alive

    def paged_decode_attention(self, layer: int, Q, O, block_table, max_blocks_per_seq: int, context_lens,
                               num_seqs: int, stream=None) -> None:
        self._check(self.lib.lkv_paged_decode_attention(self.h, layer, _ptr(Q), _ptr(O), _ptr(block_table),
                                                        max_blocks_per_seq, _ptr(context_lens), num_seqs,
                                                        _stream(stream)))

    # ------------------------------------------------------------------ ordering and statistics
    def stream_wait_event(self, layer: int, ev: int, stream=None) -> None:
        self._check(self.lib.lkv_stream_wait_event(self.h, layer, ev, _stream(stream)))

    def event_synchronize(self, layer: int, ev: int) -> None:
        self._check(self.lib.lkv_event_synchronize(self.h, layer, ev))

    def set_profiling(self, on: bool) -> None:
        self._check(self.lib.lkv_set_profiling(self.h, int(bool(on))))

    def paged_decode_attention_static(self, layer: int, Q, O, block_table, max_blocks_per_seq: int, context_lens,
                                      num_seqs: int, stream=None) -> None:
        self._check(self.lib.lkv_paged_decode_attention_static(self.h, layer, _ptr(Q), _ptr(O), _ptr(block_table),
                                                               max_blocks_per_seq, _ptr(context_lens), num_seqs,
                                                               _stream(stream)))

    def reserve_decode_workspace(self, num_seqs: int, max_blocks_per_seq: int) -> None:
        self._check(self.lib.lkv_reserve_decode_workspace(self.h, num_seqs, max_blocks_per_seq))

    def get_stats(self) -> dict:
        s = LkvStats()
        self._check(self.lib.lkv_get_stats(self.h, ctypes.byref(s), ctypes.sizeof(s)))
        return {n: getattr(s, n) for n, _ in LkvStats._fields_}
