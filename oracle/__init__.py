"""CPU oracle for the per-module ADMM structured-pruning path (STRUPRUNE).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 numpy restatement of
what the method computes (strp_oracle.py), plus the FFN iteration once more in plain fp64 torch
with its token sums accumulated chunk by chunk (strp_oracle_torch.py, pinned to the numpy
form), for modules that numpy cannot hold.  It shares no code with the HIP library and must never be
imported by the product path: only tests, the smoke check and the CPU-baseline leg of
the benchmark may use it.
"""
