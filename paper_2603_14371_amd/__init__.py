"""MI355X-native mixed action+decode attention over a shared, paged prefix KV cache.

The product path is the C-ABI library `liboxy.so` (HIP kernels for gfx950 and the
host block pool) plus the thin ctypes binding in `binding`.  `synth` only draws
seeded inputs and workload traces and is importable without the library.
"""
__all__ = ["binding", "synth", "harness"]
