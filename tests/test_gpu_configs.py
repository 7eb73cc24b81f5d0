"""Parity at the shapes of the workload configurations that fit the oracle whole or need the module loop.

* OPT-125m shape (d=768, f=3072, T=65536, 12 heads of 64): one FFN module free-running for three iterations
  against the oracle's admm_step (whole tensors), and the 12 x 64 head variant against the oracle's head_prune.
* OPT-1.3B shape (24 layers, d=2048, f=8192, T=262144): the softmax allocation for the temperature grid
  {0.5, 1, 2} over L=24 layers of n=8192 units, with the energies of three real modules at the full token count
  (the other layers' energies are seeded multiples of those), then the per-module ADMM on the three real modules
  with the allocated widths and the summed loss per temperature.
* Module streaming: three OPT-125m-shaped modules from pinned host memory through the side-stream staging onto
  the one resident state, each checked against the oracle, device memory independent of the module count.

The sampled full-size checks of the larger shapes live in test_gpu_fullsize.py.
"""
import numpy as np
import pytest
import torch

from oracle import strp_oracle as orc
from paper_2510_03246_amd import inputs, stream, strp

pytestmark = pytest.mark.gpu

TOL_F = 2e-3
TOL_J = 1e-3
TIE = 1e-6
ALPHA = BETA = 1.0
DELTA = 0.01


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def mask_mismatch_outside_ties(score64, mask_gpu, k, rel=TIE):
    mask_o, _, tau = orc.select_topk(score64, k)
    diff = np.nonzero(mask_o != mask_gpu)[0]
    return [int(j) for j in diff if abs(score64[j] - tau) > rel * abs(tau)]


# ---------------------------------------------------------------------------------------------------------
# OPT-125m shape, whole
# ---------------------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def small_run():
    cfg = inputs.CONFIGS["opt125m"]
    k = cfg.f - int(round(cfg.rbar * cfg.f))
    m = inputs.make_ffn_module(cfg, 0, 0, "cuda")
    ctx = strp.Context(0)
    mod = strp.FFNModule(ctx, m["W1hat"], m["W2hat"], m["X"], cfg.T, k_max=k)
    p = strp.Params(ALPHA, BETA, DELTA, strp.WANDA, 0, k, 0)       # Alg. 1 ordering: mask chosen at iteration 1
    mod.init(p)
    assert ctx.poll() == strp.OK
    st = orc.module_init(*(m[n].double().cpu().numpy() for n in ("W1hat", "W2hat", "X")), delta=DELTA)
    yield dict(cfg=cfg, k=k, m=m, ctx=ctx, mod=mod, p=p, st=st)
    ctx.close()


def test_config2_init_whole(small_run):
    mod, st, cfg = small_run["mod"], small_run["st"], small_run["cfg"]
    for name, ref in (("Z0", st.Z0), ("Z", st.Z0), ("A", st.A0), ("Y", st.Y)):
        assert rel_fro(getattr(mod, name)[:, :cfg.T].cpu().numpy(), ref) < 1e-5, name
    assert rel_fro(mod.H.cpu().numpy(), st.H) < 2e-6
    sc = mod.scalars.cpu().numpy()
    assert np.isclose(sc[0], st.lam1, rtol=1e-6) and np.isclose(sc[1], st.lam2, rtol=1e-6)


@pytest.mark.parametrize("it", [0, 1, 2])
def test_config2_free_running_iteration(small_run, it):
    """One more iteration on both sides (the three cases run in order on the same state)."""
    mod, st, k, p = small_run["mod"], small_run["st"], small_run["k"], small_run["p"]
    assert mod.state.iter == it, "the iterations of this test must run in order"
    rep = mod.step(p)
    terms = orc.admm_step(st, k, ALPHA, BETA, orc.WANDA, select=(it == 0))
    assert rep.status == strp.OK and rep.s == k
    if it == 0:
        assert not mask_mismatch_outside_ties(st.score, mod.mask.cpu().numpy(), k)
        assert np.array_equal(mod.idx[:k].cpu().numpy().astype(np.int64), st.idx)
        assert float(rep.tau) == np.float32(st.tau)
    got = np.array(rep.terms[:])
    assert np.all(np.abs(got - terms) <= TOL_J * terms), (it, got, terms)
    assert abs(rep.J_ridge - terms.sum()) <= TOL_J * terms.sum()
    assert abs(rep.J - terms[:3].sum()) <= TOL_J * terms[:3].sum()


def test_config2_free_running_state(small_run):
    """After the three iterations: the mask, both weight matrices and both auxiliaries, whole."""
    mod, st, cfg, k = small_run["mod"], small_run["st"], small_run["cfg"], small_run["k"]
    assert mod.state.iter == 3
    assert np.array_equal(mod.mask.cpu().numpy(), st.mask)
    err = {}
    for name in ("W1", "W2"):
        err[name] = rel_fro(getattr(mod, name).cpu().numpy(), getattr(st, name))
    for name in ("Z", "A"):
        err[name] = rel_fro(getattr(mod, name)[:, :cfg.T].cpu().numpy(), getattr(st, name))
    assert max(err.values()) < TOL_F, err
    pruned = st.mask == 0
    assert not mod.W1.cpu().numpy()[pruned].any() and not mod.W2.cpu().numpy()[:, pruned].any()


def test_config2_head_variant(small_run):
    """12 heads of 64 channels at T = 65536: head scores, kept heads and the refitted W_O against the oracle, whole."""
    cfg, ctx = small_run["cfg"], small_run["ctx"]
    d, g, T = cfg.d, cfg.d_head, cfg.T
    assert (cfg.heads, g) == (12, 64)
    m = inputs.make_head_module(cfg, 0, 0, "cuda")
    WO, Cm = m["WOhat"], m["C"]
    kh = cfg.heads - int(round(cfg.rbar * cfg.heads))
    ref = orc.head_prune(WO.double().cpu().numpy(), Cm[:, :T].double().cpu().numpy(), g, kh, DELTA)
    score = torch.empty(cfg.heads, dtype=torch.float32, device="cuda")
    energies = torch.zeros(1, dtype=torch.float64, device="cuda")
    ctx.strp_score_alloc(Cm, T, strp.WANDA, score, energies, 0, 1, group=g, What=WO)
    assert np.allclose(score.cpu().numpy(), ref["score"], rtol=1e-6)
    assert np.isclose(energies.item(), orc.layer_energy(ref["score"]), rtol=1e-6)
    mask, idx, tau = ctx.strp_mask_topk(score, kh, g)
    assert np.array_equal(mask.cpu().numpy(), ref["mask"])
    assert np.array_equal(idx.cpu().numpy().astype(np.int64), ref["idx"])
    Y = torch.from_numpy(ref["Y"]).float().cuda().contiguous()      # the dense target is an input of the refit
    G = ctx.strp_gram(Cm, T, idx=idx)
    W = torch.empty((d, d), device="cuda")
    ctx.strp_refit(strp.SIDE_FC2, G, ref["lam"], Y, Cm, T, idx, W)
    assert ctx.poll() == strp.OK
    assert rel_fro(G.cpu().numpy(), orc.gram(Cm[:, :T].double().cpu().numpy(), ref["idx"])) < 2e-6
    assert rel_fro(W.cpu().numpy(), ref["WO"]) < TOL_F
    off = np.ones(d, dtype=bool)
    off[ref["idx"]] = False
    assert not W.cpu().numpy()[:, off].any()


# ---------------------------------------------------------------------------------------------------------
# module streaming (pinned host -> side stream -> resident state)
# ---------------------------------------------------------------------------------------------------------
def test_streamed_modules_match_the_oracle_and_memory_stays_one_module():
    """Three OPT-125m-shaped modules (8192 of the tokens, so that the oracle's three runs stay short) are pinned on the
    host, staged on the side stream while the previous module iterates, bound to the one resident state, initialised
    and iterated twice.  Every module's mask, weights, auxiliaries and objective match the oracle run on that module,
    and the allocator's peak after the first module is the peak after the last."""
    cfg = inputs.with_tokens(inputs.CONFIGS["opt125m"], 8192)
    k = cfg.f - int(round(cfg.rbar * cfg.f))
    n_modules, iters = 3, 2
    torch.cuda.synchronize()
    base = torch.cuda.memory_allocated()                       # whatever other tests of this process still hold
    host = [stream.pin(inputs.make_ffn_module(cfg, layer, 0, "cpu")) for layer in range(n_modules)]
    ctx = strp.Context(0)
    streamer = stream.ModuleStreamer(host)
    first = streamer.stage[0]
    mod = strp.FFNModule(ctx, first["W1hat"], first["W2hat"], first["X"], cfg.T, k_max=k)
    p = strp.Params(ALPHA, BETA, DELTA, strp.WANDA, 0, k, 0)
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    peaks, results = [], []
    for layer, buf in streamer:
        mod.rebind_inputs(buf["W1hat"], buf["W2hat"], buf["X"])
        mod.init(p)
        for it in range(iters):
            rep = mod.step(p)
            assert rep.status == strp.OK
        # results are copied out before the next module overwrites the resident state
        results.append(dict(J=rep.J_ridge, mask=mod.mask.cpu().numpy().copy(),
                            **{n: getattr(mod, n).cpu().numpy().copy() for n in ("W1", "W2")},
                            **{n: getattr(mod, n)[:, :cfg.T].cpu().numpy().copy() for n in ("Z", "A")}))
        torch.cuda.synchronize()
        peaks.append(torch.cuda.max_memory_allocated())
    assert peaks[0] == peaks[-1], peaks                       # no growth with the number of modules
    resident = sum(t.numel() * t.element_size() for t in (mod.Z, mod.A, mod.Z0, mod.Y, mod.W1, mod.W2, mod.H, mod.cholH,
                                                          mod.cache, ctx.ws))
    assert peaks[-1] - base < resident + streamer.staging_bytes + (64 << 20)
    ctx.close()
    for layer, res in enumerate(results):
        hm = host[layer]
        st = orc.module_init(*(hm[n].double().numpy() for n in ("W1hat", "W2hat", "X")), delta=DELTA)
        for it in range(iters):
            terms = orc.admm_step(st, k, ALPHA, BETA, orc.WANDA, select=(it == 0))
        assert not mask_mismatch_outside_ties(st.score, res["mask"], k), layer
        assert abs(res["J"] - terms.sum()) <= TOL_J * terms.sum(), layer
        err = {n: rel_fro(res[n], getattr(st, n)) for n in ("W1", "W2", "Z", "A")}
        assert max(err.values()) < TOL_F, (layer, err)


# ---------------------------------------------------------------------------------------------------------
# OPT-1.3B shape: temperature grid over L = 24 layers of n = 8192 units
# ---------------------------------------------------------------------------------------------------------
def _f64_row_sumsq(t, T, chunk=1024):
    out = torch.empty(t.shape[0], dtype=torch.float64, device=t.device)
    for r0 in range(0, t.shape[0], chunk):
        out[r0:r0 + chunk] = (t[r0:r0 + chunk, :T].double() ** 2).sum(dim=1)
    return out


def test_config3_temperature_sweep():
    free, _ = torch.cuda.mem_get_info()
    if free < 70e9:
        pytest.skip("needs about 70 GB of free device memory")
    cfg = inputs.CONFIGS["opt1.3b"]
    L, n, T, rbar = cfg.L, cfg.f, cfg.T, cfg.rbar
    assert (L, n, cfg.temperatures) == (24, 8192, (0.5, 1.0, 2.0))
    real = (0, 1, 2)
    K = 2
    ctx = strp.Context(0)
    mods_in = []
    for layer in real:
        m = inputs.make_ffn_module(cfg, layer, 0, "cuda")
        # different activation scales so that the layers' energies differ (re-rounded to the storage dtype: both
        # sides see the same tensor)
        m["X"] = (m["X"].float() * (1.0 + 0.25 * layer)).to(m["X"].dtype).contiguous()
        mods_in.append(m)
    mod = strp.FFNModule(ctx, mods_in[0]["W1hat"], mods_in[0]["W2hat"], mods_in[0]["X"], T)
    energies = torch.zeros(L, dtype=torch.float64, device="cuda")
    n_units = torch.full((L,), n, dtype=torch.int32, device="cuda")
    p0 = strp.Params(ALPHA, BETA, DELTA, strp.WANDA, 0, 1, 0)
    # ---- energies of the three real modules at the full token count, each against fp64 sums of its own state
    for layer, m in zip(real, mods_in):
        mod.rebind_inputs(m["W1hat"], m["W2hat"], m["X"])
        mod.init(p0)
        ctx.strp_score_alloc(mod.A, T, strp.WANDA, mod.score, energies, layer, L, n2=mod.n2)
        assert ctx.poll() == strp.OK
        n2 = (m["W2hat"].double() ** 2).sum(dim=0)
        ref_score = orc.unit_scores(_f64_row_sumsq(mod.A, T).cpu().numpy(), n2.cpu().numpy(), 0, 0, 0, orc.WANDA)
        assert np.allclose(mod.score.cpu().numpy(), ref_score, rtol=2e-6)
        assert np.isclose(energies[layer].item(), orc.layer_energy(ref_score), rtol=2e-6)
    # ---- the other 21 layers: seeded multiples of the real energies (harness; both sides read the same vector)
    rng = np.random.default_rng(3)
    e = energies.cpu().numpy()
    for layer in range(len(real), L):
        e[layer] = e[layer % len(real)] * rng.uniform(0.6, 1.8)
    energies.copy_(torch.from_numpy(e))
    r_out = torch.empty(L, dtype=torch.float64, device="cuda")
    npr = torch.empty(L, dtype=torch.int32, device="cuda")
    totals = {}
    for temp in cfg.temperatures:
        # the allocation runs on the device through strp_score_alloc (scoring layer 0 again leaves its energy as it was)
        m = mods_in[0]
        mod.rebind_inputs(m["W1hat"], m["W2hat"], m["X"])
        mod.init(p0)
        ctx.strp_score_alloc(mod.A, T, strp.WANDA, mod.score, energies, 0, L, n2=mod.n2, n_units=n_units, rbar=rbar,
                             temperature=temp, rmax=0.95, r_out=r_out, nprune_out=npr)
        assert ctx.poll() == strp.OK
        assert np.array_equal(energies.cpu().numpy(), e)
        r_ref, npr_ref = orc.softmax_allocation(e, np.full(L, n), rbar, temp)
        assert np.allclose(r_out.cpu().numpy(), r_ref, rtol=1e-12, atol=1e-15)
        assert np.array_equal(npr.cpu().numpy().astype(np.int64), npr_ref)
        assert int(npr_ref.sum()) == int(round(float((r_ref * n).sum())))
        # ---- per-module ADMM with the allocated widths on the three real modules
        losses = []
        for layer, m in zip(real, mods_in):
            k = n - int(npr_ref[layer])
            p = strp.Params(ALPHA, BETA, DELTA, strp.WANDA, 0, k, 0)
            if layer != 0:
                mod.rebind_inputs(m["W1hat"], m["W2hat"], m["X"])
                mod.init(p)
            for it in range(K):
                rep = mod.step(p)
            assert rep.status == strp.OK and rep.s == k
            assert int(mod.mask.sum().item()) == k
            losses.append(rep.J_ridge)
            if layer == real[-1]:
                # the reported loss against its definition in fp64 on the state the device holds
                idx = mod.idx[:k].long()
                W2S, W1S = mod.W2[:, idx].double(), mod.W1[idx].double()
                t1 = t2 = t3 = 0.0
                for t0 in range(0, T, 16384):
                    t1_ = min(T, t0 + 16384)
                    A, Z = mod.A[:, t0:t1_].double(), mod.Z[:, t0:t1_].double()
                    t1 += float(((mod.Y[:, t0:t1_].double() - W2S @ A[idx]) ** 2).sum().item())
                    t2 += float(((A - torch.relu(Z)) ** 2).sum().item())
                    Z1 = torch.zeros_like(Z)
                    Z1[idx] = W1S @ m["X"][:, t0:t1_].double()
                    t3 += float(((Z - Z1) ** 2).sum().item())
                    del A, Z, Z1
                J = (ALPHA * t1 + BETA * t2 + ALPHA * t3 + ALPHA * rep.lam2 * float((mod.W2.double() ** 2).sum().item())
                     + ALPHA * rep.lam1 * float((mod.W1.double() ** 2).sum().item())) / T
                assert abs(rep.J_ridge - J) <= TOL_J * J, (temp, rep.J_ridge, J)
        totals[temp] = float(np.sum(losses))
    assert all(np.isfinite(v) and v > 0 for v in totals.values())
    best = min(totals, key=totals.get)
    assert best in cfg.temperatures          # T* is the argmin of the three totals; its value has no further pin
    ctx.close()
