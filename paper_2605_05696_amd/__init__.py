"""MI355X-native cache-hit re-attachment path for an MLA position-independent KV cache.

``binding`` is the thin ctypes layer over the C-ABI library (``include/irm.h``);
``workloads`` holds the seeded synthetic input generators.  Nothing here falls
back to a CPU implementation: using the binding without the built HIP library
raises.
"""
__all__ = ["binding", "workloads", "build"]
