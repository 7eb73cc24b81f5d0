"""Alg. 1 end to end on one GPU, composed from the library's entry points: the layers' energies once, then per
temperature of the grid the softmax sparsity allocation (Lemma 2, Alg. 1 steps 1-2) -> per-module ADMM with the
allocated widths (Alg. 3, FFN function) -> summed loss; the best temperature is the argmin of the totals (Alg. 1 step 5).

Orchestration only: every number is produced by libstrp.so.  One module state is resident; the modules' inputs are
re-bound to it one after another, so the device memory is that of one module whatever the depth of the model.  The
modules are either dicts of device tensors, or dicts of PINNED HOST tensors (stream.pin), which travel to the device
through stream.ModuleStreamer (two staging sets, copies on a side stream beside the previous module's iterations).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch

from . import stream, strp


@dataclass
class TemperatureResult:
    temperature: float
    energies: list            # I_l, one per module
    r: list                   # allocated pruned fraction per module
    nprune: list              # units pruned per module
    losses: list              # augmented objective J + ridge terms of each module after its iterations
    total: float
    pruned: list = field(default_factory=list)   # per module (mask, W1, W2) clones, kept for the best temperature only


def _walk(modules, device):
    """Yield (layer, dict of device tensors) in layer order."""
    if modules[0]["X"].is_cuda:
        yield from enumerate(modules)
    else:
        yield from stream.ModuleStreamer(modules, device=device)


def prune_model(ctx: strp.Context, modules, T: int, rbar: float, temperatures, iters: int, alpha: float = 1.0,
                beta: float = 1.0, delta: float = 0.01, mode: int = strp.WANDA, reselect: int = 0, rmax: float = 0.95,
                keep_weights: bool = False, on_module=None):
    """modules: list of dicts with "W1hat" [f x d], "W2hat" [d x f], "X" [d x ld] of equal shapes, all on the device or
    all in pinned host memory.  on_module(temperature, layer, module, report), if given, is called after a module's last
    iteration while its state is still resident (to copy out what the caller wants to keep).
    Returns ({temperature: TemperatureResult}, best_temperature)."""
    modules = list(modules)
    L = len(modules)
    assert L > 0
    f = modules[0]["W1hat"].shape[0]
    dev = ctx.device
    mod = None
    n_units = torch.full((L,), f, dtype=torch.int32, device=dev)
    energies = torch.zeros(L, dtype=torch.float64, device=dev)
    p_init = strp.Params(alpha, beta, delta, mode, reselect, 1, 0)
    full = mode != strp.WANDA

    # ---- the energies do not depend on the temperature: every module is initialised and scored once
    for layer, m in _walk(modules, dev):
        if mod is None:
            mod = strp.FFNModule(ctx, m["W1hat"], m["W2hat"], m["X"], T)
        else:
            mod.rebind_inputs(m["W1hat"], m["W2hat"], m["X"])
        mod.init(p_init)
        ctx.strp_score_alloc(mod.A, T, mode, mod.score, energies, layer, L, n2=mod.n2, Z=mod.Z if full else None,
                             Z0=mod.Z0 if full else None)
    status = ctx.poll()
    if status != strp.OK:
        raise strp.StrpError(status, "scoring failed")
    e_h = energies.cpu().tolist()
    results = {}
    best = None
    for temp in temperatures:
        r_out, npr = ctx.strp_alloc_softmax(energies, n_units, rbar, float(temp), rmax)
        r_h, npr_h = r_out.cpu().tolist(), [int(v) for v in npr.cpu().tolist()]
        losses, kept = [None] * L, [None] * L
        for layer, m in _walk(modules, dev):
            k = f - npr_h[layer]
            p = strp.Params(alpha, beta, delta, mode, reselect, k, 0)
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
            if on_module is not None:
                on_module(temp, layer, mod, rep)
        res = TemperatureResult(float(temp), e_h, r_h, npr_h, losses, float(sum(losses)))
        results[temp] = res
        if best is None or res.total < results[best].total:
            if best is not None:
                results[best].pruned = []
            res.pruned = kept if keep_weights else []
            best = temp
    return results, best
