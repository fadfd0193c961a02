"""Two-Pass softmax (arXiv 2001.04438) for MI355X: hand-written HIP behind a C ABI.

The kernels live in csrc/ and are reached through the thin ctypes binding in
binding.py; workloads.py holds the seeded synthetic input recipes.
"""
__all__ = ["binding", "workloads", "buildlib"]
