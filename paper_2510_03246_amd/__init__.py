"""MI355X-native per-module ADMM structured pruning (STRUPRUNE hot path).

The compute path lives in the HIP library `libstrp.so` (sources under csrc/); `strp`
is the ctypes binding with the same entry-point names.  Importing this package does not
load the library; the first call through `strp` does, and fails loudly if it is missing.
"""
