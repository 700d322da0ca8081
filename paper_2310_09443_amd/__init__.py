"""G10 tensor-vitality analysis and migration planning on MI355X (HIP, gfx950).

`traces` holds the synthetic workloads; `binding` is the thin ctypes layer over
the C-ABI library built from `csrc/` (it raises if the library is missing).
"""
__all__ = ["traces", "binding"]
