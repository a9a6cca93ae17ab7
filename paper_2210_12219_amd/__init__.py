"""Exact partition-and-placement search (minimum bottleneck latency) on MI355X.

`workloads` holds the seeded synthetic inputs; `binding` is the thin ctypes layer over the
C-ABI library built from csrc/ (loaded on first use, never at import of this package).
"""
__all__ = ["workloads", "binding"]
