"""Sparse/dense gradient aggregation hot path of Parallax (arXiv 1808.02621) for MI355X.

Importing the package loads nothing native.  ``paper_1808_02621_amd.px`` is the
ctypes binding of the HIP library (it raises if the library is not built);
``paper_1808_02621_amd.inputs`` holds the seeded synthetic input generators,
which contain none of the method's arithmetic.
"""

__all__ = ["inputs", "px"]
