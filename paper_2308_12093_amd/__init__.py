"""MI355X-native GCN / GAT layer forward + backward with adaptive operator
reordering and caching (arXiv 2308.12093), behind a C-ABI library.

Importing the package loads nothing native: ``paper_2308_12093_amd.binding``
loads the HIP library on first use and raises if it has not been built
(there is no CPU fallback); ``paper_2308_12093_amd.synth`` makes the seeded
synthetic inputs and needs NumPy only.
"""

__all__ = ["binding", "synth", "build"]
