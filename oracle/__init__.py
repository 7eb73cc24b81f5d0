"""CPU oracle for the per-module ADMM structured-pruning path (STRUPRUNE).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 numpy restatement of
what the method computes.  It shares no code with the HIP library and must never be
imported by the product path: only tests, the smoke check and the CPU-baseline leg of
the benchmark may use it.
"""
