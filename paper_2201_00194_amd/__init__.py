"""MI355X-native batched scoring of candidate programs by per-family tree-ensemble cost
models, with per-program statement sums and a per-family top-k cut.

Importing the package loads nothing native; `paper_2201_00194_amd.api` binds the C-ABI
library and raises if it has not been built.
"""
__all__ = ["workloads"]
