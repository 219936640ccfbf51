"""MI355X-native projection-pruning hot path (Mosaic, arXiv 2504.06323).

`synth` manufactures seeded inputs; `prune` is the thin binding over the C-ABI
library built from `csrc/`.  Importing the package does not load the library:
that happens on the first call, and fails loudly if it has not been built.
"""
__all__ = ["synth", "prune"]
