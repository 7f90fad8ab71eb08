"""Reslim ViT forward under TILES (ORBIT-2, Sec. 4.1-4.2) for one MI355X.

`workloads` holds the seeded synthetic inputs; `binding` is the thin ctypes layer
over the C-ABI library built from `csrc/` (imported lazily: it needs the built
shared object and, for compute calls, a GPU).
"""
__all__ = ["workloads", "binding"]
