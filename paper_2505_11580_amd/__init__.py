"""fipa: factorized Invariant Point Attention for MI355X (gfx950).

`binding` is the thin ctypes layer over the C-ABI library (include/fipa.h);
`workloads` holds the seeded synthetic input generators.  Importing the package
loads nothing native; `binding.lib()` does, and fails loudly if the library is
not built.
"""
__all__ = ["binding", "workloads", "build"]
