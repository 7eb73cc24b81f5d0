"""The accuracy-for-passes table of the design notes, reproducible: free-running ADMM iterations with fp16 planes
dropped product by product through strp_set_product_planes.  Not a pytest file (its name keeps it out of collection);
it needs an MI355X and, for part "oracle", minutes of host time.

    python tests/precision_table.py oracle  ITERS [short]    # OPT-125m-shaped module, whole, against the oracle
    python tests/precision_table.py self WORKLOAD ITERS [short]   # any workload, against the library's own 3-pass run
    python tests/precision_table.py device WORKLOAD ITERS [short] # opt1.3b / opt6.7b against the oracle's chunked torch
                                                                  # form in fp64 on the GPU (its own trajectory)

Both parts select once and then hold the mask (reselect = 0), so that every variant follows the same kept set and the
figures are errors of the arithmetic, not of a diverged selection.  "short" runs the combined variants only.
Columns: relative Frobenius error of W1, W2, Z, A after the last iteration, relative error of the objective, number of
mask entries that differ, and (part "self") milliseconds of one more iteration in that setting.
"""
import os
import sys
import time

import numpy as np
import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from oracle import strp_oracle as orc                      # noqa: E402
from oracle import strp_oracle_torch as ort                # noqa: E402
from paper_2510_03246_amd import inputs, strp              # noqa: E402

NAMES = ["GRAM", "RHS2", "RHS1", "RESID", "AUPD", "ZUPD"]
SINGLE = [("base", [])]
for prod, opts in ((0, [(1, 1), (2, 1)]), (1, [(1, 2), (2, 1), (1, 1)]), (2, [(1, 1)]), (3, [(1, 2), (2, 1), (1, 1)]),
                   (4, [(1, 2), (2, 1), (1, 1)]), (5, [(1, 1)])):
    for o in opts:
        SINGLE.append((f"{NAMES[prod]}{o[0]}x{o[1]}", [(prod, o)]))
SINGLE.append(("ALL1x1", [(p, (1, 1)) for p in range(6)]))
# "null": nothing dropped, one element of Z and of A moved by one part in 1e6 before the first iteration
COMBINED = [("base", []), ("null", "perturb"),
            ("4x(2x1)", [(0, (2, 1)), (1, (2, 1)), (3, (2, 1)), (4, (2, 1))]),
            ("4x(1x2)", [(0, (2, 1)), (1, (1, 2)), (3, (1, 2)), (4, (1, 2))]),
            ("G22+3x21", [(1, (2, 1)), (3, (2, 1)), (4, (2, 1))]),
            ("RES+AUP21", [(3, (2, 1)), (4, (2, 1))]),
            ("ALL1x1", [(p, (1, 1)) for p in range(6)])]


def rel(a, b):
    num = den = 0.0
    step = max(1, (1 << 27) // max(a.shape[1], 1))
    for r0 in range(0, a.shape[0], step):
        x, y = a[r0:r0 + step].double(), b[r0:r0 + step].double()
        num += float(((x - y) ** 2).sum().item())
        den += float((y ** 2).sum().item())
    return (num / max(den, 1e-300)) ** 0.5


def run(ctx, mod, p, iters, setting):
    for prod in range(6):
        ctx.set_product_planes(prod, 2, 2)
    perturb = setting == "perturb"
    for prod, (a, b) in ([] if perturb else setting):
        ctx.set_product_planes(prod, a, b)
    mod.init(p)
    if perturb:
        mod.Z[7, 11] *= 1.000001
        mod.A[9, 13] *= 1.000001
    rep = None
    for _ in range(iters):
        rep = mod.step(p)
    assert rep.status == strp.OK
    return rep


def against_oracle(iters, variants):
    cfg = inputs.CONFIGS["opt125m"]
    k = cfg.f - int(round(cfg.rbar * cfg.f))
    m = inputs.make_ffn_module(cfg, 0, 0, "cuda")
    st = orc.module_init(*(m[n].double().cpu().numpy() for n in ("W1hat", "W2hat", "X")))
    t0 = time.time()
    terms = None
    for it in range(iters):
        terms = orc.admm_step(st, k, 1.0, 1.0, orc.WANDA, select=(it == 0))
        print("oracle iteration", it, flush=True)
    print(f"oracle: {time.time() - t0:.0f} s", flush=True)
    ref = {n: torch.from_numpy(getattr(st, n)).cuda() for n in ("W1", "W2", "Z", "A")}
    j_ref = float(np.sum(terms))
    ctx = strp.Context(0)
    mod = strp.FFNModule(ctx, m["W1hat"], m["W2hat"], m["X"], cfg.T, k_max=k)
    p = strp.Params(1.0, 1.0, 0.01, strp.WANDA, 0, k, 0)
    print(f"opt125m whole against the oracle, {iters} iterations")
    print(f"{'variant':12s} {'W1':>9s} {'W2':>9s} {'Z':>9s} {'A':>9s} {'J':>9s} maskdiff")
    for name, setting in variants:
        rep = run(ctx, mod, p, iters, setting)
        e = {n: rel(getattr(mod, n)[:, :ref[n].shape[1]], ref[n]) for n in ref}
        md = int((mod.mask.cpu().numpy() != st.mask).sum())
        print(f"{name:12s} {e['W1']:9.2e} {e['W2']:9.2e} {e['Z']:9.2e} {e['A']:9.2e} {abs(rep.J_ridge - j_ref) / j_ref:9.2e} {md}",
              flush=True)
    for prod in range(6):
        ctx.set_product_planes(prod, 2, 2)
    ctx.close()


def against_device_fp64(workload, iters, variants):
    cfg = inputs.CONFIGS[workload]
    k = cfg.f - int(round(cfg.rbar * cfg.f))
    m = inputs.make_ffn_module(cfg, 0, 0, "cuda")
    t0 = time.time()
    st = ort.module_init(m["W1hat"], m["W2hat"], m["X"], cfg.T)
    terms = None
    for it in range(iters):
        terms = ort.admm_step(st, k, 1.0, 1.0, select=(it == 0))
    torch.cuda.synchronize()
    print(f"fp64 reference on the device: {time.time() - t0:.0f} s", flush=True)
    ref = {n: getattr(st, n) for n in ("W1", "W2", "Z", "A")}
    j_ref = float(np.sum(terms))
    ctx = strp.Context(0)
    mod = strp.FFNModule(ctx, m["W1hat"], m["W2hat"], m["X"], cfg.T, k_max=k)
    p = strp.Params(1.0, 1.0, 0.01, strp.WANDA, 0, k, 0)
    print(f"{workload} against fp64 on the device, {iters} iterations")
    print(f"{'variant':12s} {'W1':>9s} {'W2':>9s} {'Z':>9s} {'A':>9s} {'J':>9s} maskdiff")
    for name, setting in variants:
        if name == "null":
            continue
        rep = run(ctx, mod, p, iters, setting)
        e = {n: rel(getattr(mod, n)[:, :ref[n].shape[1]], ref[n]) for n in ref}
        md = int((mod.mask.cpu().numpy() != st.mask).sum())
        print(f"{name:12s} {e['W1']:9.2e} {e['W2']:9.2e} {e['Z']:9.2e} {e['A']:9.2e} {abs(rep.J_ridge - j_ref) / j_ref:9.2e} {md}",
              flush=True)
    for prod in range(6):
        ctx.set_product_planes(prod, 2, 2)
    ctx.close()


def against_itself(workload, iters, variants):
    cfg = inputs.CONFIGS[workload]
    k = cfg.f - int(round(cfg.rbar * cfg.f))
    m = inputs.make_ffn_module(cfg, 0, 0, "cuda")
    ctx = strp.Context(0)
    mod = strp.FFNModule(ctx, m["W1hat"], m["W2hat"], m["X"], cfg.T, k_max=k)
    p = strp.Params(1.0, 1.0, 0.01, strp.WANDA, 0, k, 0)
    rep = run(ctx, mod, p, iters, [])
    ref = {n: getattr(mod, n).clone() for n in ("W1", "W2", "Z", "A")}
    ref_mask, j_ref = mod.mask.clone(), rep.J_ridge
    print(f"{workload} against the run with every plane, {iters} iterations")
    print(f"{'variant':12s} {'W1':>9s} {'W2':>9s} {'Z':>9s} {'A':>9s} {'J':>9s} maskdiff  ms/step")
    for name, setting in variants:
        if name == "base":
            continue
        rep = run(ctx, mod, p, iters, setting)
        e = {n: rel(getattr(mod, n), ref[n]) for n in ref}
        md = int((mod.mask != ref_mask).sum().item())
        torch.cuda.synchronize()
        t0 = time.time()
        mod.step(p, report=False)
        torch.cuda.synchronize()
        ms = (time.time() - t0) * 1e3
        print(f"{name:12s} {e['W1']:9.2e} {e['W2']:9.2e} {e['Z']:9.2e} {e['A']:9.2e} {abs(rep.J_ridge - j_ref) / j_ref:9.2e} {md:6d}  {ms:7.1f}",
              flush=True)
    for prod in range(6):
        ctx.set_product_planes(prod, 2, 2)
    ctx.close()


if __name__ == "__main__":
    short = sys.argv[-1] == "short"
    args = sys.argv[1:-1] if short else sys.argv[1:]
    variants = COMBINED if short else SINGLE
    if args[0] == "oracle":
        against_oracle(int(args[1]), variants)
    elif args[0] == "self":
        against_itself(args[1], int(args[2]), variants)
    elif args[0] == "device":
        against_device_fp64(args[1], int(args[2]), variants)
    else:
        sys.exit(__doc__)
