"""msGeMM (look-up-table GeMM, arxiv 2310.06178) for AMD MI355X / gfx950.

``paper_2310_06178_amd.inputs``  seeded synthetic inputs (no method arithmetic)
``paper_2310_06178_amd.binding`` ctypes binding of the C-ABI HIP library

Nothing is imported eagerly: the binding loads ``libmsgemm.so`` on first use and
raises if it has not been built (there is no CPU fallback).
"""
__all__ = ["inputs", "binding"]
