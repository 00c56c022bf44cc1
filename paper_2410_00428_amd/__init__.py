"""Layer-wise paged KV cache hot path for AMD MI355X (gfx950).

The product is the C-ABI library ``liblkv.so`` (sources under ``csrc/``, declarations in
``include/lkv.h``); ``binding`` is the thin ctypes layer over it and ``workloads`` holds
the seeded input generators.  Nothing is imported eagerly so that ``workloads`` can be
used without the compiled library.
"""
__all__ = ["binding", "workloads", "build"]
