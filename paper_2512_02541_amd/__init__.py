"""Subsampled global attention (AVGGT, Sec. 4.3) for AMD MI355X (gfx950).

``paper_2512_02541_amd.binding`` is the thin ctypes layer over the C-ABI library
``libagg.so`` (declared in ``include/agg.h``); ``paper_2512_02541_amd.inputs``
draws the seeded synthetic workloads.  Importing the package loads nothing: the
shared library is opened on first use and a missing library is an error, never a
fallback.
"""

__all__ = ["binding", "inputs", "build"]
