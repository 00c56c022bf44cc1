"""CPU oracle for the layer-wise paged KV cache -- TEST INFRASTRUCTURE, not the product.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py``
may import this package.  It never imports the HIP package, and the HIP package never
imports it.
"""
