"""MI355X-native verification step of RAPID (retrieval-augmented speculative decoding).

``paper_2502_20330_amd.binding`` is the thin ctypes layer over the C-ABI
library ``librapid.so`` (hand-written gfx950 kernels); ``workloads`` holds the
seeded synthetic input generators.  Nothing here computes on the CPU: without
the built library every call raises.
"""
__all__ = ["binding", "workloads"]
