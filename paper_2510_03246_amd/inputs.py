"""Seeded synthetic module inputs (weights and calibration activations).

This module only draws random tensors of the shapes and distributions of the workloads;
it contains none of the pruning arithmetic.  Both the HIP path and the test oracle consume
the tensors produced here (generated once, then handed to each side).

Stand-in for the paper's calibration protocol (128 segments of 2048 tokens through an OPT
decoder): activations are Gaussian with a few heavy-tailed or amplified outlier channels,
weights are N(0, 0.02^2) rounded to the configuration's storage dtype.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    L: int            # decoder layers (modules per family)
    d: int            # model width
    f: int            # FFN hidden width
    heads: int        # attention heads (0: FFN only)
    T: int            # calibration tokens
    dtype: str        # "f32" | "bf16" storage of X and the pre-trained weights
    outlier: str      # "x20" (amplified Gaussian channels) | "t3" (Student-t, nu = 3)
    n_outlier: int
    rbar: float       # target pruned fraction
    K: int            # ADMM iterations
    temperatures: tuple = (1.0,)

    @property
    def d_head(self):
        return self.d // self.heads if self.heads else 0


CONFIGS = {
    "tiny": WorkloadConfig("tiny", 2, 64, 256, 0, 512, "f32", "x20", 2, 0.5, 10),
    "opt125m": WorkloadConfig("opt125m", 12, 768, 3072, 12, 32 * 2048, "bf16", "t3", 8, 0.5, 20),
    "opt1.3b": WorkloadConfig("opt1.3b", 24, 2048, 8192, 32, 128 * 2048, "bf16", "t3", 21, 0.6, 20,
                              (0.5, 1.0, 2.0)),
    "opt6.7b": WorkloadConfig("opt6.7b", 32, 4096, 16384, 32, 128 * 2048, "bf16", "t3", 41, 0.7, 20),
    "opt30b": WorkloadConfig("opt30b", 48, 7168, 28672, 56, 128 * 2048, "bf16", "t3", 72, 0.7, 20),
}


def with_tokens(cfg: WorkloadConfig, T: int) -> WorkloadConfig:
    """Same workload with a different number of calibration tokens."""
    return replace(cfg, T=T)


def torch_dtype(name: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _gen(seed: int, layer: int, tensor_id: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1_000_003 + layer) * 101 + tensor_id)
    return g


def _activations(rows: int, cfg: WorkloadConfig, seed: int, layer: int, tensor_id: int, device,
                 ld: int | None = None):
    """[rows, T] activations in the storage dtype; row stride ld >= T (padding zero-filled)."""
    T = cfg.T
    ld = T if ld is None else ld
    dt = torch_dtype(cfg.dtype)
    out = torch.zeros((rows, ld), dtype=dt, device=device)
    gsel = _gen(seed, layer, tensor_id + 50, "cpu")
    special = torch.randperm(rows, generator=gsel)[: cfg.n_outlier].tolist()
    g = _gen(seed, layer, tensor_id, device)
    chunk = max(1, min(rows, (1 << 26) // max(T, 1)))
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        x = torch.randn((r1 - r0, T), generator=g, device=device, dtype=torch.float32)
        for ch in special:
            if r0 <= ch < r1:
                if cfg.outlier == "x20":
                    x[ch - r0] *= 20.0
                else:
                    w = torch.randn((3, T), generator=g, device=device, dtype=torch.float32)
                    x[ch - r0] = x[ch - r0] / torch.sqrt((w * w).mean(dim=0))
        out[r0:r1, :T] = x.to(dt)
    return out


def _weight(rows: int, cols: int, cfg: WorkloadConfig, seed: int, layer: int, tensor_id: int, device):
    g = _gen(seed, layer, tensor_id, device)
    w = torch.randn((rows, cols), generator=g, device=device, dtype=torch.float32) * 0.02
    return w.to(torch_dtype(cfg.dtype))


def make_ffn_module(cfg: WorkloadConfig, layer: int = 0, seed: int = 0, device="cpu", ld: int | None = None):
    """Pre-trained fc1/fc2 weights and the fc1 input of one FFN module.

    Returns dict(W1hat [f,d], W2hat [d,f], X [d,ld] with X[:, :T] valid).
    """
    return dict(
        W1hat=_weight(cfg.f, cfg.d, cfg, seed, layer, 1, device),
        W2hat=_weight(cfg.d, cfg.f, cfg, seed, layer, 2, device),
        X=_activations(cfg.d, cfg, seed, layer, 3, device, ld),
    )


def make_head_module(cfg: WorkloadConfig, layer: int = 0, seed: int = 0, device="cpu", ld: int | None = None):
    """Output-projection weights and concatenated head outputs of one attention module."""
    return dict(
        WOhat=_weight(cfg.d, cfg.d, cfg, seed, layer, 11, device),
        C=_activations(cfg.d, cfg, seed, layer, 12, device, ld),
    )


def synthetic_state(rows: int, T: int, seed: int, device, relu: bool = False, ld: int | None = None):
    """[rows, ld] fp32 stand-in for an ADMM auxiliary variable (used by kernel-level tests)."""
    g = _gen(seed, 0, 21, device)
    ld = T if ld is None else ld
    out = torch.zeros((rows, ld), dtype=torch.float32, device=device)
    x = torch.randn((rows, T), generator=g, device=device, dtype=torch.float32)
    out[:, :T] = torch.relu(x) if relu else x
    return out
