"""exat: multi-replica tensor compression Y_p = X x1 U_p x2 V_p x3 W_p on MI355X (gfx950).

The compute lives in the C-ABI library built from csrc/ (see include/exat.h);
`paper_2311_13693_amd.exat` is the thin ctypes binding over it and
`paper_2311_13693_amd.workloads` the seeded synthetic-input recipes.
Nothing is imported eagerly so that the input recipes can be used without the
GPU library being present.
"""
__all__ = ["exat", "workloads"]
