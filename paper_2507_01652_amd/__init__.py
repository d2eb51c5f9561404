"""MI355X-native LASAD hot path: linear attention with Spatial-Aware Decay.

The compute lives in ``liblasad.so`` (hand-written HIP for gfx950, C ABI declared
in ``include/lasad.h``); ``binding`` is a thin ctypes layer over it and
``workloads`` generates the seeded synthetic inputs.  Importing the package loads
nothing heavy; the library is opened on first use and its absence is an error
(there is no CPU fallback).
"""

__all__ = ["binding", "workloads", "build"]
