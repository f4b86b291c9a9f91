"""BalanceRoute route-step path for MI355X (gfx950).

`workloads` draws seeded synthetic inputs; `binding` is the thin ctypes layer over
the C-ABI HIP library in `csrc/`.  Importing the package loads neither.
"""
__all__ = ["workloads", "binding"]
