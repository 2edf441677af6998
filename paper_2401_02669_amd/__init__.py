"""DistAttention decode hot path for MI355X (gfx950).

``paper_2401_02669_amd.distattn`` is the Python binding over the C-ABI library
``libdistattn.so`` (HIP kernels); ``paper_2401_02669_amd.synth`` makes seeded
synthetic workloads.  Importing the package loads nothing native: the binding
loads the library on first use and raises if it has not been built.
"""
__all__ = ["distattn", "synth"]
