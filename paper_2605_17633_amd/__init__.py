"""MI355X-native structured-sparse SAM ViT encoder block (SparseSAM, arXiv 2605.17633).

The compute path is a C-ABI HIP library (``csrc/``, header ``include/ssam.h``);
``binding`` marshals arguments into it and ``inputs`` draws seeded synthetic
arrays.  Importing the package does not load the library; the first call into
``binding`` does, and raises if it has not been built.
"""
__all__ = ["inputs", "binding"]
