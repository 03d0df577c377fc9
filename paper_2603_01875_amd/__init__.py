"""libkdloss: full-vocabulary knowledge-distillation loss (forward + backward)
as hand-written gfx950 kernels behind a C ABI.

Importing the package loads nothing native; `paper_2603_01875_amd.kdloss`
loads the shared library on first use and raises if it has not been built.
"""
__all__ = ["inputs", "kdloss"]
