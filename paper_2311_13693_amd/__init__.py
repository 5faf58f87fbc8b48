"""exat: multi-replica tensor compression Y_p = X x1 U_p x2 V_p x3 W_p on MI355X (gfx950).

The compute lives in the C-ABI library built from csrc/ (see include/exat.h);
`paper_2311_13693_amd.exat` is the thin ctypes binding over it.  Nothing is
imported eagerly.  The seeded synthetic-input recipes that tests and benchmark
feed to both this library and the CPU oracle live outside the package, in the
top-level module `workloads`.
"""
__all__ = ["exat"]
