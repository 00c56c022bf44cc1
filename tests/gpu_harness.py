"""Shared plumbing of the GPU parity tests: device buffers via torch, calls via the C ABI binding,
expected values via the CPU oracle.  torch is used for memory and streams only."""
from __future__ import annotations

import numpy as np
import torch

from oracle import layerkv_oracle as orc
from paper_2410_00428_amd import binding as lkv
from paper_2410_00428_amd import workloads as wl

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    """Upload raw storage (float32, int32, int64 or bf16 bit patterns as int16)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).to(DEV)


def to_host(t: torch.Tensor, dtype: str) -> np.ndarray:
    """Download a tensor of the config's storage type and widen it to float32."""
    a = t.cpu().numpy()
    if dtype == "bf16":
        return wl.bf16_bits_to_f32(a.view(np.uint16))
    return a.astype(np.float32)


def empty_like_storage(shape, dtype: str) -> torch.Tensor:
    return torch.empty(tuple(shape), dtype=torch.float32 if dtype == "f32" else torch.int16, device=DEV)


def zero_pool(shape: wl.KVShape, num_blocks: int) -> torch.Tensor:
    return torch.zeros(num_blocks * shape.block_bytes, dtype=torch.uint8, device=DEV)


def pool_as_oracle_view(pool: torch.Tensor, o: orc.LayerKVOracle) -> np.ndarray:
    return pool.cpu().numpy().view(o.np_dtype).reshape(o.pool.shape)


def make_pair(shape: wl.KVShape, num_blocks: int, free_order=None, **kw):
    """A library context on a zeroed torch-owned pool and an oracle with the same free list."""
    pool = zero_pool(shape, num_blocks)
    c = lkv.LKV(shape.num_layers, shape.num_q_heads, shape.num_kv_heads, shape.head_dim, shape.block_size,
                num_blocks, shape.dtype, pool=pool, **kw)
    scales = {k: kw[k] for k in ("k_scale", "v_scale") if k in kw}
    o = orc.LayerKVOracle(shape.num_layers, shape.num_q_heads, shape.num_kv_heads, shape.head_dim,
                          shape.block_size, num_blocks, shape.dtype, **scales)
    if free_order is not None:
        c.pool_reset(free_order)
        o.pool_reset(free_order)
    return c, o, pool


def pinned_bytes(n: int) -> torch.Tensor:
    return torch.empty(max(n, 1), dtype=torch.uint8, pin_memory=True)


# ------------------------------------------------------------------ tolerances (written out here, used by every test)
def check_attention(got: np.ndarray, ref: np.ndarray, dtype: str, sigma_v: float = 1.0, what: str = "") -> None:
    """got, ref: [..., d].  fp32: row-wise max error <= 1e-5 * row max of the reference (against the
    fp64-accumulated oracle).  bf16 (fp32 accumulation): the stated 2e-2 absolute + 1e-2 relative
    bound, plus the binding row-wise and tensor-level L2 bounds (the stated one is vacuous for
    outputs of magnitude ~1e-2)."""
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref)
    if dtype == "f32":
        rowmax = np.abs(ref).max(axis=-1, keepdims=True)
        bad = err > 1e-5 * rowmax + 1e-30
        assert not bad.any(), f"{what}: fp32 row-wise rel err {np.max(err / (rowmax + 1e-30)):.3e} > 1e-5"
        return
    assert (err <= 2e-2 + 1e-2 * np.abs(ref)).all(), f"{what}: bf16 abs/rel bound violated, max err {err.max():.3e}"
    rows_g = got.reshape(-1, got.shape[-1])
    rows_r = ref.reshape(-1, ref.shape[-1])
    num = np.linalg.norm(rows_g - rows_r, axis=1)
    den = np.linalg.norm(rows_r, axis=1)
    lim = 1e-2 * den + 1e-3 * sigma_v
    assert (num <= lim).all(), f"{what}: row-wise L2 bound violated: worst ratio {np.max(num / lim):.3f}"
    tot = np.linalg.norm(rows_g - rows_r) / max(np.linalg.norm(rows_r), 1e-30)
    assert tot <= 5e-3, f"{what}: tensor-level relative L2 error {tot:.3e} > 5e-3"
