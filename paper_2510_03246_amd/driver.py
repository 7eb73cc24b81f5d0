"""Alg. 1 end to end on one GPU, composed from the library's entry points: per temperature of the grid, the layers'
energies -> softmax sparsity allocation (Lemma 2, Alg. 1 steps 1-2) -> per-module ADMM with the allocated widths
(Alg. 3, FFN function) -> summed loss; the best temperature is the argmin of the totals (Alg. 1 step 5).

Orchestration only: every number is produced by libstrp.so.  One module state is resident; the modules' inputs are
re-bound to it one after another (device tensors, or host modules handed over through stream.ModuleStreamer), so the
device memory is that of one module whatever the depth of the model.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch

from . import strp


@dataclass
class TemperatureResult:
    temperature: float
    energies: list            # I_l, one per module
    r: list                   # allocated pruned fraction per module
    nprune: list              # units pruned per module
    losses: list              # augmented objective J + ridge terms of each module after its iterations
    total: float
    pruned: list = field(default_factory=list)   # per module (mask, W1, W2) clones, kept for the best temperature only


def prune_model(ctx: strp.Context, modules, T: int, rbar: float, temperatures, iters: int, alpha: float = 1.0,
                beta: float = 1.0, delta: float = 0.01, mode: int = strp.WANDA, reselect: int = 0, rmax: float = 0.95,
                keep_weights: bool = False):
    """modules: sequence of dicts with device tensors "W1hat" [f x d], "W2hat" [d x f], "X" [d x ld] of equal shapes
    (or any iterable that yields such dicts each time it is iterated, e.g. a list of stream.ModuleStreamer items
    materialised by the caller).  Returns ({temperature: TemperatureResult}, best_temperature)."""
    modules = list(modules)
    L = len(modules)
    assert L > 0
    m0 = modules[0]
    f = m0["W1hat"].shape[0]
    dev = m0["X"].device
    mod = strp.FFNModule(ctx, m0["W1hat"], m0["W2hat"], m0["X"], T)
    n_units = torch.full((L,), f, dtype=torch.int32, device=dev)
    energies = torch.zeros(L, dtype=torch.float64, device=dev)
    r_out = torch.empty(L, dtype=torch.float64, device=dev)
    npr = torch.empty(L, dtype=torch.int32, device=dev)
    p_init = strp.Params(alpha, beta, delta, mode, reselect, 1, 0)
    full = mode != strp.WANDA

    def score(layer, **alloc):
        m = modules[layer]
        mod.rebind_inputs(m["W1hat"], m["W2hat"], m["X"])
        mod.init(p_init)
        ctx.strp_score_alloc(mod.A, T, mode, mod.score, energies, layer, L, n2=mod.n2, Z=mod.Z if full else None,
                             Z0=mod.Z0 if full else None, **alloc)

    # the energies do not depend on the temperature: every layer is scored once, the last one again per temperature
    # because the allocation runs inside a scoring call
    for layer in range(L - 1):
        score(layer)
    results = {}
    best = None
    for temp in temperatures:
        score(L - 1, n_units=n_units, rbar=rbar, temperature=float(temp), rmax=rmax, r_out=r_out, nprune_out=npr)
        status = ctx.poll()
        if status != strp.OK:
            raise strp.StrpError(status, "allocation failed")
        e_h, r_h, npr_h = energies.cpu().tolist(), r_out.cpu().tolist(), [int(v) for v in npr.cpu().tolist()]
        losses, kept = [None] * L, [None] * L
        for layer in [L - 1] + list(range(L - 1)):   # the last module is resident and initialised: it goes first
            k = f - npr_h[layer]
            p = strp.Params(alpha, beta, delta, mode, reselect, k, 0)
            if layer != L - 1:
                m = modules[layer]
                mod.rebind_inputs(m["W1hat"], m["W2hat"], m["X"])
                mod.init(p)
            rep = None
            for it in range(iters):
                rep = mod.step(p)
                if rep.status != strp.OK:
                    raise strp.StrpError(rep.status, f"module {layer}, iteration {it}")
            losses[layer] = rep.J_ridge
            if keep_weights:
                kept[layer] = (mod.mask.clone(), mod.W1.clone(), mod.W2.clone())
        res = TemperatureResult(float(temp), e_h, r_h, npr_h, losses, float(sum(losses)))
        results[temp] = res
        if best is None or res.total < results[best].total:
            if best is not None:
                results[best].pruned = []
            res.pruned = kept if keep_weights else []
            best = temp
    return results, best
