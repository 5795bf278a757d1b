"""srft-kv: fused SRFT -> lambda -> per-group int4 KV-cache quantizer for MI355X (gfx950).

The compute lives in the HIP library ``libsrft_kv.so`` (C ABI declared in
``include/srft_kv.h``); ``binding`` is the thin ctypes layer over it and
``workloads`` draws the seeded synthetic caches.  Importing this package does
not load the library; the first use of ``binding`` does, and raises if the
library has not been built.
"""
__all__ = ["binding", "workloads", "build"]
