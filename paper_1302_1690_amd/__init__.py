"""Whole-image MaxPooling-CNN segmentation training on MI355X (gfx950).

`paper_1302_1690_amd.mpcnn` is the thin binding over the C-ABI library
(`libmpcnn.so`, built from `csrc/`); `paper_1302_1690_amd.workloads` holds the
seeded synthetic input generators.  Importing the package loads nothing native;
the binding loads the library on first use and raises if it has not been built.
"""
__all__ = ["workloads", "mpcnn"]
