"""Float64 CPU oracle of the CLIP contrastive loss and its DisCo decomposition.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and its
Python binding) imports, links or calls this package; only tests/, the smoke
check and the benchmark's cpu_baseline leg do.  It shares no code with the GPU
path.  Every function is pinned by tests/test_oracle_*pins.py (closed forms, finite
differences, brute force, a library autograd transcription of the paper's
Alg. 1, and the paper's rank-sum equivalence); none is "parity unpinned".
"""
