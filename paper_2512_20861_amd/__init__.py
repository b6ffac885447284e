"""MI355X-native forward pass of block low-rank (Monarch, BLAST) linear layers.

The product is the C-ABI library built from csrc/ (see include/blr.h); `binding` exposes its
entry points to Python, `roofline` holds the closed-form traffic/FLOP model used by the benchmark.
"""
from . import binding  # noqa: F401
