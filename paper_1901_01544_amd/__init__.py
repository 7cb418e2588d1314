"""MI355X-native importance-weighted-pruning compression step (arXiv 1901.01544).

``paper_1901_01544_amd.iwp`` is the thin binding over the C-ABI HIP library;
``paper_1901_01544_amd.workloads`` generates the seeded synthetic inputs.
Nothing is loaded at import time: the HIP library is opened on first use and a
missing library is an error, never a fallback.
"""
__all__ = ["iwp", "workloads"]
