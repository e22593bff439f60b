"""Tiled mixed-precision spGEMM (C = A*B) for AMD MI355X (gfx950).

``inputs`` draws the synthetic workloads; ``tsp`` is the thin binding over the
C-ABI library built from ``csrc/``.  Importing the package does not load the
library; every ``tsp`` call does and raises if it has not been built.
"""
from . import inputs  # noqa: F401

__all__ = ["inputs"]
