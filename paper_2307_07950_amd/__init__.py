"""MI355X-native SelSync per-step hot path (gradient-change tracking, fused local
SGD update, K-replica parameter aggregation) behind a C-ABI library.

Importing the package does not load the HIP library; ``paper_2307_07950_amd.binding``
does, and fails loudly if it has not been built."""
__all__ = ["workloads"]
