"""MI355X-native SparseMoE expert hot path (FastSparseMoE, Section 3.1 / Algorithm 1).

``workloads`` draws synthetic inputs; ``binding`` is the thin ctypes layer over
the C-ABI library built from ``csrc/``.  Nothing is loaded at import time.
"""
__all__ = ["workloads", "binding", "build"]
