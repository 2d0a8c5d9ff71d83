"""Shared-KV decode attention for MI355X (gfx950): hand-written HIP kernels behind a C ABI.

`paper_2410_18517_amd.binding` is the thin ctypes layer over libkvs.so (argument
marshalling only); `paper_2410_18517_amd.inputs` holds the seeded synthetic workloads.
There is no CPU fallback: using the binding without the built library raises.
"""
__all__ = ["binding", "inputs"]
