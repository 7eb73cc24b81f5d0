"""ctypes binding of libstrp_bench.so: the sustained rate of the fp16 matrix-core instruction the GEMMs use.

A measurement aid of bench.py (reported as "mfma_ceiling"), no part of the method and not in libstrp.so.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libstrp_bench.so")
_lib = None


def mfma_rate(kind: int, milliseconds: float = 200.0) -> float:
    """TFLOP/s of the fp16 matrix-core instruction on the current stream.  kind 0: v_mfma_f32_16x16x32_f16 on constant
    register operands; 2: random fp16 values in the registers; 1: the pipelined GEMM's inner loop without its memory
    side (fragments re-read from LDS); 3: kind 1 on v_mfma_f32_32x32x16_f16 (same flops, same LDS traffic)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2510_03246_amd.build`")
        _lib = C.CDLL(LIB_PATH)
        _lib.strp_bench_mfma_rate.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32, C.c_double,
                                              C.POINTER(C.c_double)]
        _lib.strp_bench_mfma_rate.restype = C.c_int
    scratch = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    out = C.c_double(0.0)
    st = _lib.strp_bench_mfma_rate(C.c_void_p(torch.cuda.current_stream().cuda_stream), C.c_void_p(scratch.data_ptr()),
                                   scratch.numel(), kind, float(milliseconds), C.byref(out))
    if st != 0:
        raise RuntimeError(f"strp_bench_mfma_rate failed with status {st}")
    return out.value
