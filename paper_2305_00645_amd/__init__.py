"""MI355X-native hot path of GTree: three-party secret-shared decision-tree training
and inference over Z_2^64 (arXiv 2305.00645).  The compute lives in the HIP library
under ``csrc/``; ``gtree`` is a thin ctypes binding with the same entry-point names;
``workloads`` holds the seeded synthetic input generators."""
