"""CPU oracle for segmented causal attention and the computation-wise partition.

TEST INFRASTRUCTURE ONLY.  Nothing under this package is part of the product: only the tests, the
smoke check and the benchmark's `cpu_baseline` leg may import it.  It shares no code with the HIP
path and never calls it.  Every function is the plain definition of the quantity, written from the
paper (Section 3.1 Eq. 3 for attention, Section 3.4 Eq. 7-8 for the partition), in fp64 / exact
integers, with no tiling, fusion or online softmax.

Pins (see tests/test_oracle_*.py): closed forms, finite differences, an independent library routine,
brute force on tiny inputs, and the paper's claim that segment-wise execution leaves results unchanged.
"""
