"""pxr — MI355X-native batched pixel-observation renderer (hot path of PixelBrax, arXiv 2502.00021).

`paper_2502_00021_amd.pxr` is the ctypes binding of the C-ABI HIP library;
`paper_2502_00021_amd.workloads` holds the seeded synthetic input generators.
Nothing is imported eagerly so that the generators stay usable without the
built library; the binding itself raises if the library is missing.
"""
__all__ = ["pxr", "workloads"]
