"""Tree-masked verification attention for MI355X (gfx950).

`workloads` draws the seeded synthetic inputs; `binding` is the thin ctypes
layer over the C-ABI library built from `csrc/` (imported lazily so that the
input generators can be used without the HIP library being present).
"""

__all__ = ["workloads", "binding"]
