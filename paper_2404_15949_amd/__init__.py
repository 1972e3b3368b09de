"""MI355X-native decode hot path of CORM (arXiv 2404.15949): ragged per-head
attention + recent-query score record + eviction + stable compaction.

``inputs`` draws the seeded synthetic workloads; ``corm`` binds the C-ABI
library built from ``csrc/``.  Importing the package does not load the
library; the binding loads it on first use and raises if it is missing.
"""
__all__ = ["inputs", "corm"]
