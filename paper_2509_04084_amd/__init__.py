"""MI355X-native LowDiff hot path: differential-checkpoint build and merge.

``paper_2509_04084_amd.lowdiff`` is the thin binding over the C-ABI HIP library
(``ld_compress_topk``, ``ld_snapshot_layer``, ``ld_merge_sparse``,
``ld_merge_dense_adam``); ``paper_2509_04084_amd.synth`` holds the seeded
synthetic workloads.  Importing the package loads nothing heavy.
"""
__all__ = ["lowdiff", "synth"]
