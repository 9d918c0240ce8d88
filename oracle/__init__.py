"""CPU oracle for the packed variable-length transformer-block step and the balanced packer.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only tests/, the smoke
check and the bench's cpu_baseline leg do.  It shares no code with the HIP path.

Everything here is the plain definition written out with numpy (fp64 by default, dtype
selectable), with no tiling, fusion, online softmax or reordering.  Pinned by the CPU tests
(tests/test_oracle_*.py): per-segment equivalence, softmax row sums, central finite differences,
closed forms of the norms / GELU / rotary, brute-force GEMM, GQA-vs-MHA replication, hand-worked
packer examples and the values the paper prints for its Fig. 2 example.

Parity unpinned: none of the functions; but the paper's printed DistRatio / GPU-day table values
cannot be reproduced (they need the paper's datasets) and are not used as pins.
"""
