"""MI355X-native range-filtered graph search over a bucketed index (GRAB-ANNS hot path).

``workloads`` makes seeded synthetic inputs (vectors, attributes, queries, ranges); ``binding`` is the thin ctypes layer over the
C-ABI library ``libgrab.so`` built from ``csrc/`` (every step of the search and append
path runs in its HIP kernels).  Nothing is loaded at import time.
"""
__all__ = ["workloads", "binding", "build"]
