"""Full-size checks: the OPT-1.3B-, OPT-6.7B- and OPT-30B-shaped modules (d=2048/4096/7168, f=4d, T=262144, 60/70/70 %
of the units pruned), each run exactly as bench.py runs it (module init, then one call of strp_admm_step with every
stage, WANDA, re-select).  At f=28672 the step's select takes the radix kernel instead of the register-resident one,
and k=8602 leaves a different ragged remainder in every product that has k as a tile dimension.

The oracle cannot run this size whole, so every stage is checked on sampled outputs that the oracle's
own functions (or its definitions) can produce one by one, teacher-forced from the state the GPU holds:
token columns for the token-parallel products, weight rows for the refits.  Token sums of length T that a
sampled output needs (a Gram matrix, a right-hand-side row) are accumulated in fp64 by torch on the
device - harness arithmetic, not the library - and the small dense solve is the oracle's (numpy).
Tolerances are those of the medium-size parity tests.
"""
import gc

import numpy as np
import pytest
import torch

from oracle import strp_oracle as orc
from paper_2510_03246_amd import inputs, strp

pytestmark = pytest.mark.gpu

TOL_F = 2e-3
TOL_J = 1e-3
ALPHA = BETA = 1.0
DELTA = 0.01


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def f64_nt(P, Q, T, chunk=16384):
    """sum_t P[:, t] Q[:, t]^T over the first T columns, accumulated in fp64 on the device."""
    out = torch.zeros((P.shape[0], Q.shape[0]), dtype=torch.float64, device=P.device)
    for t0 in range(0, T, chunk):
        t1 = min(T, t0 + chunk)
        out += P[:, t0:t1].double() @ Q[:, t0:t1].double().T
    return out


NEED_BYTES = {"opt1.3b": 50e9, "opt6.7b": 140e9, "opt30b": 225e9}


@pytest.fixture(scope="module", params=["opt1.3b", "opt6.7b", "opt30b"])
def run(request):
    gc.collect()
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < NEED_BYTES[request.param]:
        pytest.skip(f"needs about {NEED_BYTES[request.param] / 1e9:.0f} GB of free device memory")
    cfg = inputs.CONFIGS[request.param]
    k = cfg.f - int(round(cfg.rbar * cfg.f))
    m = inputs.make_ffn_module(cfg, 0, 0, "cuda")
    ctx = strp.Context(0)
    mod = strp.FFNModule(ctx, m["W1hat"], m["W2hat"], m["X"], cfg.T, k_max=k)
    params = strp.Params(ALPHA, BETA, DELTA, strp.WANDA, 1, k, 0)
    mod.init(params)
    torch.cuda.synchronize()
    assert ctx.poll() == strp.OK
    rng = np.random.default_rng(0)
    cols = np.sort(rng.choice(cfg.T, size=4, replace=False))
    cols[-1] = cfg.T - 1                                   # the ragged end of the last tile
    init = {n: getattr(mod, n)[:, cols].double().cpu().numpy() for n in ("Z0", "Z", "A", "Y")}
    lam = (float(mod.scalars[0].item()), float(mod.scalars[1].item()))
    rep = mod.step(params)
    torch.cuda.synchronize()
    assert rep.status == strp.OK
    res = dict(cfg=cfg, k=k, m=m, mod=mod, cols=cols, init=init, lam=lam, rep=rep)
    yield res
    ctx.close()
    res.clear()
    del mod, m, ctx
    gc.collect()
    torch.cuda.empty_cache()


def test_init_columns(run):
    """Z0 = W1hat X, A0 = ReLU(Z0), Y = W2hat A0 on sampled token columns; the ridge constants."""
    m, cols, init, cfg = run["m"], run["cols"], run["init"], run["cfg"]
    W1 = m["W1hat"].double().cpu().numpy()
    W2 = m["W2hat"].double().cpu().numpy()
    Xc = m["X"][:, cols].double().cpu().numpy()
    st = orc.module_init(W1, W2, Xc)                        # per-column quantities do not depend on the other tokens
    assert rel_fro(init["Z0"], st.Z0) < 1e-5
    assert rel_fro(init["Z"], st.Z0) < 1e-5
    assert rel_fro(init["A"], st.A0) < 1e-5
    assert rel_fro(init["Y"], st.Y) < 1e-5
    mod = run["mod"]
    sumsq = 0.0
    for r0 in range(0, cfg.f, 1024):
        sumsq += float((torch.relu(mod.Z0[r0:r0 + 1024, :cfg.T]).double() ** 2).sum().item())
    assert abs(run["lam"][1] - DELTA * sumsq / cfg.f) <= 1e-6 * run["lam"][1]
    trH = float((m["X"][:, :cfg.T].double() ** 2).sum().item())
    assert abs(run["lam"][0] - DELTA * trH / cfg.d) <= 1e-6 * run["lam"][0]


def test_scores_and_mask(run):
    """WANDA scores of sampled units from their activation rows; the mask is the oracle's top-k of the scores."""
    mod, cfg, k, m = run["mod"], run["cfg"], run["k"], run["m"]
    rng = np.random.default_rng(1)
    units = rng.choice(cfg.f, size=16, replace=False)
    A0 = np.maximum(mod.Z0[units, :cfg.T].double().cpu().numpy(), 0.0)
    n2 = (m["W2hat"][:, units].double().cpu().numpy() ** 2).sum(axis=0)
    ref = orc.unit_scores(np.einsum("jt,jt->j", A0, A0), n2, 0, 0, 0, orc.WANDA)
    score = mod.score.cpu().numpy()
    assert np.allclose(score[units], ref, rtol=1e-6, atol=0)
    mask_o, idx_o, tau_o = orc.select_topk(score, k)
    assert np.array_equal(mod.mask.cpu().numpy(), mask_o)
    assert np.array_equal(mod.idx[:k].cpu().numpy().astype(np.int64), idx_o)
    assert run["rep"].s == k and float(run["rep"].tau) == np.float32(tau_o)


def test_refits_sampled_rows(run):
    """Rows of the refitted weights against the ridge normal equations solved by the oracle's solver."""
    mod, cfg, k, m, (lam1, lam2) = run["mod"], run["cfg"], run["k"], run["m"], run["lam"]
    T = cfg.T
    idx = mod.idx[:k].long()
    keep = mod.mask.bool()
    assert not bool(mod.W2[:, ~keep].any()) and not bool(mod.W1[~keep, :].any())   # pruned units are exactly zero
    # the refits of the first iteration see A = ReLU(Z0), Z = Z0
    AS = torch.relu(mod.Z0[idx, :T])
    G = f64_nt(AS, AS, T).cpu().numpy()
    rows = torch.tensor([0, cfg.d // 3, cfg.d - 1], device="cuda")
    R2 = f64_nt(mod.Y[rows, :T], AS, T).cpu().numpy()
    ref2 = np.linalg.solve(G + lam2 * np.eye(k), R2.T).T
    got2 = mod.W2[rows][:, idx].cpu().numpy()
    assert rel_fro(got2, ref2) < TOL_F / 4
    del AS
    X = m["X"]
    H = f64_nt(X, X, T).cpu().numpy()
    units = idx[torch.tensor([0, k // 2, k - 1], device="cuda")]
    R1 = f64_nt(mod.Z0[units, :T], X, T).cpu().numpy()
    ref1 = np.linalg.solve(H + lam1 * np.eye(cfg.d), R1.T).T
    got1 = mod.W1[units].cpu().numpy()
    assert rel_fro(got1, ref1) < TOL_F / 4


def test_a_and_z_updates_sampled_columns(run):
    """The a-update and z-update on sampled token columns, teacher-forced with the weights the GPU refitted."""
    mod, cfg, k, m, cols, init = run["mod"], run["cfg"], run["k"], run["m"], run["cols"], run["init"]
    idx = mod.idx[:k].long().cpu().numpy()
    W2S = mod.W2[:, idx].double().cpu().numpy()
    # pruned columns of W2 are zero (checked above), so the f x f system of the a-update decouples: the oracle's
    # function on the kept block, and ReLU(Z) on the other rows
    A_ref = orc.a_update(W2S, init["Y"], init["Z0"][idx], ALPHA, BETA)
    A_gpu = mod.A[:, cols].double().cpu().numpy()
    assert rel_fro(A_gpu[idx], A_ref) < TOL_F
    pruned = np.setdiff1d(np.arange(cfg.f), idx)
    assert np.array_equal(A_gpu[pruned], np.maximum(init["Z0"][pruned], 0.0))
    W1S = mod.W1[idx].double().cpu().numpy()
    Xc = m["X"][:, cols].double().cpu().numpy()
    Z_ref = orc.z_update(W1S, Xc, A_gpu[idx], ALPHA, BETA)
    Z_gpu = mod.Z[:, cols].double().cpu().numpy()
    assert rel_fro(Z_gpu[idx], Z_ref) < TOL_F
    Zp_ref = orc.z_update(np.zeros((len(pruned), 1)), np.zeros((1, len(cols))), A_gpu[pruned], ALPHA, BETA)
    assert np.allclose(Z_gpu[pruned], Zp_ref, rtol=1e-6, atol=0)
    # whole pruned rows: ReLU of the previous z, and its half
    rows = torch.from_numpy(pruned[[0, len(pruned) // 2, -1]]).cuda()
    a_rows = torch.relu(mod.Z0[rows, :cfg.T])
    assert torch.equal(mod.A[rows, :cfg.T], a_rows)
    assert torch.allclose(mod.Z[rows, :cfg.T], a_rows * (BETA / (ALPHA + BETA)), rtol=1e-6, atol=0)


def test_objective(run):
    """The reported objective against its definition evaluated in fp64 on the state the GPU holds."""
    mod, cfg, k, m, rep, (lam1, lam2) = run["mod"], run["cfg"], run["k"], run["m"], run["rep"], run["lam"]
    T = cfg.T
    idx = mod.idx[:k].long()
    W2S = mod.W2[:, idx].double()
    W1S = mod.W1[idx].double()
    keep = mod.mask.bool()
    t1 = t2 = t3 = 0.0
    chunk = 8192
    for t0 in range(0, T, chunk):
        t1_ = min(T, t0 + chunk)
        A = mod.A[:, t0:t1_].double()
        Z = mod.Z[:, t0:t1_].double()
        t1 += float(((mod.Y[:, t0:t1_].double() - W2S @ A[idx]) ** 2).sum().item())
        t2 += float(((A - torch.relu(Z)) ** 2).sum().item())
        Z1 = torch.zeros_like(Z)
        Z1[idx] = W1S @ m["X"][:, t0:t1_].double()
        t3 += float(((Z - Z1) ** 2).sum().item())
        del A, Z, Z1
    terms = np.array([ALPHA * t1, BETA * t2, ALPHA * t3,
                      ALPHA * lam2 * float((mod.W2.double() ** 2).sum().item()),
                      ALPHA * lam1 * float((mod.W1.double() ** 2).sum().item())]) / T
    got = np.array(list(rep.terms))
    assert np.all(np.abs(got - terms) <= TOL_J * np.maximum(terms, 1e-12)), (got, terms)
    assert abs(rep.J_ridge - terms.sum()) <= TOL_J * terms.sum()
    assert abs(rep.J - terms[:3].sum()) <= TOL_J * terms[:3].sum()
    assert keep.sum().item() == k


def test_gain_and_lemma_scores_on_moved_state(run):
    """After one iteration Z != Z0 and A != A0: the three-tensor token sums (GAIN, LEMMA) at full size."""
    mod, cfg, m = run["mod"], run["cfg"], run["m"]
    ctx = mod.ctx
    rng = np.random.default_rng(2)
    units = rng.choice(cfg.f, size=12, replace=False)
    rows = torch.from_numpy(units).cuda()
    A, Z, Z0 = (getattr(mod, n)[rows, :cfg.T].double().cpu().numpy() for n in ("A", "Z", "Z0"))
    W2u = m["W2hat"][:, rows].double().cpu().numpy()
    sums = orc.unit_sums(A, np.maximum(Z0, 0.0), Z, Z0, W2u)
    score = torch.empty(cfg.f, dtype=torch.float32, device="cuda")
    energies = torch.zeros(1, dtype=torch.float64, device="cuda")
    for mode_gpu, mode_ref in ((strp.GAIN, orc.GAIN), (strp.LEMMA, orc.LEMMA)):
        ctx.strp_score_alloc(mod.A, cfg.T, mode_gpu, score, energies, 0, 1, Z=mod.Z, Z0=mod.Z0, n2=mod.n2)
        assert ctx.poll() == strp.OK
        ref = orc.unit_scores(*sums, mode_ref)
        assert np.allclose(score.cpu().numpy()[units], ref, rtol=2e-6, atol=0)
        assert np.isclose(energies.item(), float(score.double().mean().item()), rtol=1e-6)


def test_gain_select_inside_a_step(run):
    """A select-only call of strp_admm_step in GAIN mode on the moved state (at f = 28672 this is the radix top-k
    kernel): the mask and the ascending index list are the oracle's top-k of the scores it computed, and sampled
    scores equal 2P - Q from fp64 token sums.  Restores what the selection overwrites."""
    mod, cfg, k, m = run["mod"], run["cfg"], run["k"], run["m"]
    saved = {n: getattr(mod, n).clone() for n in ("mask", "idx", "score", "scalars")}
    saved_cached = mod.state.sums_cached
    mod.step(strp.Params(ALPHA, BETA, DELTA, strp.GAIN, 1, k, strp.STAGE_SELECT))
    assert mod.ctx.poll() == strp.OK
    score = mod.score.cpu().numpy()
    mask_o, idx_o, tau_o = orc.select_topk(score, k)
    assert np.array_equal(mod.mask.cpu().numpy(), mask_o)
    assert np.array_equal(mod.idx[:k].cpu().numpy().astype(np.int64), idx_o)
    rng = np.random.default_rng(4)
    units = rng.choice(cfg.f, size=8, replace=False)
    rows = torch.from_numpy(units).cuda()
    A, Z, Z0 = (getattr(mod, n)[rows, :cfg.T].double().cpu().numpy() for n in ("A", "Z", "Z0"))
    sums = orc.unit_sums(A, np.maximum(Z0, 0.0), Z, Z0, m["W2hat"][:, rows].double().cpu().numpy())
    assert np.allclose(score[units], orc.unit_scores(*sums, orc.GAIN), rtol=2e-6, atol=0)
    for n, t in saved.items():
        getattr(mod, n).copy_(t)
    mod.state.s = k
    mod.state.sums_cached = saved_cached


def test_second_selection_from_cached_sums(run):
    """The iteration kept the scoring sums of every row (pruned rows: the pass that writes them; kept rows: the epilogues
    of the a- and z-update products): the next selection streams nothing and gives the scores and the mask of a selection
    that streams every row, and sampled scores equal n2_j * sum_t A_jt^2 of the state (restores what a selection
    overwrites)."""
    mod, cfg, k = run["mod"], run["cfg"], run["k"]
    assert mod.state.sums_cached & 1
    saved = {n: getattr(mod, n).clone() for n in ("mask", "idx", "score")}
    saved_scalars = mod.scalars.clone()
    sel = strp.Params(ALPHA, BETA, DELTA, strp.WANDA, 1, k, strp.STAGE_SELECT)
    mod.ctx.profile_enable(True)
    mod.step(sel)
    assert not any(n.startswith("row_sums") for n in mod.ctx.profile_read())      # nothing was streamed
    mod.ctx.profile_enable(False)
    score_cached, mask_cached = mod.score.clone(), mod.mask.clone()
    mod.state.sums_cached = 0
    mod.step(sel)
    assert mod.state.sums_cached & 1
    assert torch.allclose(score_cached, mod.score, rtol=1e-6, atol=0)
    assert torch.equal(mask_cached, mod.mask)
    rng = np.random.default_rng(3)
    units = np.concatenate([rng.choice(cfg.f, size=6, replace=False), mod.idx[:3].cpu().numpy()])
    rows = torch.from_numpy(units).cuda().long()
    g = (mod.A[rows, :cfg.T].double() ** 2).sum(dim=1)
    ref = (mod.n2[rows] * g).cpu().numpy()
    assert np.allclose(score_cached[rows].cpu().numpy(), ref, rtol=2e-6, atol=0)
    for n, t in saved.items():
        getattr(mod, n).copy_(t)
    mod.scalars.copy_(saved_scalars)
    mod.state.s = k


def test_head_variant_at_full_width(run):
    """Head pruning of an output projection at the configuration's width (32 x 64, 32 x 128 or 56 x 128 channels, T = 262144): head scores, the
    kept heads and sampled rows of the refitted W_O against fp64 (uses the fixture's context and workspace)."""
    cfg, ctx = run["cfg"], run["mod"].ctx
    d, g, T = cfg.d, cfg.d // cfg.heads, cfg.T
    m = inputs.make_head_module(cfg, 0, 0, "cuda")
    WO, Cm = m["WOhat"], m["C"]
    kh = cfg.heads - int(round(cfg.rbar * cfg.heads))
    score = torch.empty(cfg.heads, dtype=torch.float32, device="cuda")
    energies = torch.zeros(1, dtype=torch.float64, device="cuda")
    ctx.strp_score_alloc(Cm, T, strp.WANDA, score, energies, 0, 1, group=g, What=WO)
    n2 = (WO.double() ** 2).sum(dim=0)
    gsum = torch.zeros(d, dtype=torch.float64, device="cuda")
    for t0 in range(0, T, 32768):
        gsum += (Cm[:, t0:min(T, t0 + 32768)].double() ** 2).sum(dim=1)
    ref_score = (n2 * gsum).view(cfg.heads, g).sum(dim=1).cpu().numpy()
    assert np.allclose(score.cpu().numpy(), ref_score, rtol=2e-6)
    mask, idx, tau = ctx.strp_mask_topk(score, kh, g)
    mo, io, to = orc.select_topk(ref_score.astype(np.float32), kh, g)
    assert np.array_equal(mask.cpu().numpy(), mo) and np.array_equal(idx.cpu().numpy().astype(np.int64), io)
    Y = torch.empty((d, Cm.shape[1]), dtype=torch.float32, device="cuda")
    for t0 in range(0, T, 32768):
        Y[:, t0:t0 + 32768] = (WO.double() @ Cm[:, t0:t0 + 32768].double()).float()
    lam = DELTA * float(gsum.sum().item()) / d
    G = ctx.strp_gram(Cm, T, idx=idx)
    W = torch.empty((d, d), device="cuda")
    ctx.strp_refit(strp.SIDE_FC2, G, lam, Y, Cm, T, idx, W)
    assert ctx.poll() == strp.OK
    li = idx.long()
    CS = Cm[li, :T]
    Gd = f64_nt(CS, CS, T).cpu().numpy()
    assert rel_fro(G.cpu().numpy(), Gd) < 1e-5
    rows = torch.tensor([0, d // 2 + 1, d - 1], device="cuda")
    R = f64_nt(Y[rows, :T], CS, T).cpu().numpy()
    ref = np.linalg.solve(Gd + lam * np.eye(li.numel()), R.T).T
    assert rel_fro(W[rows][:, li].cpu().numpy(), ref) < TOL_F / 4
    off = torch.ones(d, dtype=torch.bool, device="cuda")
    off[li] = False
    assert not bool(W[:, off].any())


def test_gain_iteration_keeps_every_rows_sums(run):
    """One full GAIN iteration with re-selection at full size (the pruned rows' pass reads Z0 as well and rides with the
    factorisation chains, the kept rows' sums come from the a/z epilogues): afterwards a selection from the cached sums
    gives the scores and the mask of a selection that streams every row of A, Z and Z0 again.  Moves the state."""
    mod, k = run["mod"], run["k"]
    rep = mod.step(strp.Params(ALPHA, BETA, DELTA, strp.GAIN, 1, k, 0))
    assert rep.status == strp.OK
    assert mod.state.sums_cached == 7
    sel = strp.Params(ALPHA, BETA, DELTA, strp.GAIN, 1, k, strp.STAGE_SELECT)
    mod.ctx.profile_enable(True)
    mod.step(sel)
    assert not any(n.startswith("row_sums") for n in mod.ctx.profile_read())
    mod.ctx.profile_enable(False)
    score_cached, mask_cached = mod.score.clone(), mod.mask.clone()
    mod.state.sums_cached = 0
    mod.step(sel)
    assert mod.ctx.poll() == strp.OK
    # 2P - Q is a difference of sums: agreement is relative to the largest score
    scale = float(mod.score.abs().max().item())
    assert float((score_cached - mod.score).abs().max().item()) <= 2e-6 * scale
    # the two masks may differ only in units whose score lies within that agreement of the threshold
    tau = float(torch.sort(mod.score, descending=True).values[k - 1].item())
    differ = (mask_cached != mod.mask).nonzero().flatten().cpu().numpy()
    assert all(abs(float(mod.score[j].item()) - tau) <= 4e-6 * scale for j in differ), differ


def test_objective_does_not_rise_on_a_fixed_mask(run):
    """Block-coordinate descent on the augmented objective (Appendix A.1: every update is the exact minimiser of its
    block): with the mask held, three more iterations at full size never raise J + ridge terms, and the pruned rows'
    pass — which at these sizes rides along with the factorisation chains — leaves its drain kernel almost nothing.
    Runs last in this module: it moves the state."""
    mod, k = run["mod"], run["k"]
    p = strp.Params(ALPHA, BETA, DELTA, strp.WANDA, 0, k, 0)
    prev = mod.step(p).J_ridge            # the mask is whatever the tests before left; it stays from here on
    mod.ctx.profile_enable(True)
    for it in range(3):
        rep = mod.step(p)
        assert rep.status == strp.OK
        assert rep.J_ridge <= prev * (1.0 + 1e-6), (it, rep.J_ridge, prev)
        prev = rep.J_ridge
    prof = mod.ctx.profile_read()
    mod.ctx.profile_enable(False)
    drain = [v for n, v in prof.items() if n == "pruned_rows_drain"]
    factor = [v for n, v in prof.items() if n == "chol_factor_f64"]
    assert drain and factor
    # the whole pass streamed by the drain alone takes several milliseconds at these sizes
    assert drain[0]["ms"] / drain[0]["launches"] < 0.25 * factor[0]["ms"] / factor[0]["launches"]
