"""MI355X-native SOAR NVFP4 weight quantization (hot path).

``paper_2605_12245_amd.binding`` is the thin ctypes view of the HIP library's
C-ABI (``include/soar.h``); ``paper_2605_12245_amd.synth`` generates the seeded
synthetic workloads.  Importing the package does not load the HIP library;
calling any entry point without it raises.
"""
__all__ = ["binding", "synth"]
