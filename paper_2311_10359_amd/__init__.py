"""FIKIT trace profiling and gap-fill evaluation on MI355X (gfx950).

`traces`  - seeded synthetic launch traces (inputs only).
`binding` - thin ctypes binding of the C-ABI library (`fikit_profile`, `fikit_gapfill`, ...);
            every step of the path runs in the library's HIP kernels.
The HIP library is loaded on first use of `binding`, not on import of the package.
"""
__all__ = ["traces", "binding"]
