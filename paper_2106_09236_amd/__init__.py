"""MI355X-native prob-sparse self-attention forward (arXiv 2106.09236, Sec. 3).

`workloads` draws the seeded synthetic inputs; `binding` is the thin ctypes
layer over the C-ABI library built from `csrc/` (loaded on first use; it
raises if the library has not been built).
"""
__all__ = ["workloads", "binding"]
