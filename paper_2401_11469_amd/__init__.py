"""MI355X-native resized tensor-parallel shard GEMMs (ZERO-resizing hot path).

``paper_2401_11469_amd.zr`` is the ctypes binding of the C-ABI HIP library;
``paper_2401_11469_amd.workloads`` holds the seeded synthetic inputs.
Nothing is imported eagerly so that the input generators stay usable on a
machine without the built library.
"""
__all__ = ["workloads", "zr"]
