"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test checks an oracle function against something other than itself: brute-force
enumeration, a library routine on a special case, a closed form, or an invariant.
"""
import itertools

import numpy as np
import pytest
import scipy.optimize

from oracle import strp_oracle as orc


def _tiny_state(seed=0, d=5, f=9, T=24, moved=True):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(d, T))
    W1 = rng.normal(size=(f, d)) * 0.5
    W2 = rng.normal(size=(d, f)) * 0.5
    st = orc.module_init(W1, W2, X, delta=0.01)
    if moved:  # move the auxiliaries away from their initial values
        st.Z = st.Z + 0.3 * rng.normal(size=st.Z.shape)
        st.A = np.maximum(st.A + 0.3 * rng.normal(size=st.A.shape), 0.0)
    return st


# ---- P1: the mask rule against brute force over all channel subsets (eq. (78)) -------
@pytest.mark.parametrize("seed,k", [(0, 4), (1, 3), (2, 6)])
def test_gain_rule_is_the_exact_subset_optimum(seed, k):
    st = _tiny_state(seed)
    bf_mask, bf_val = orc.brute_force_mask(k, st.X, st.Z, st.Z0, st.A, st.A0, st.W2hat)
    score = orc.module_scores(st, orc.GAIN)
    mask, idx, tau = orc.select_topk(score, k)
    assert np.array_equal(mask, bf_mask)
    # and the objective gap of flipping one unit equals its score (independent evaluation)
    ones = np.ones(score.shape[0])
    full = orc.separable_objective(ones, st.X, st.Z, st.Z0, st.A, st.A0, st.W2hat)
    for j in range(score.shape[0]):
        M = ones.copy()
        M[j] = 0.0
        drop = orc.separable_objective(M, st.X, st.Z, st.Z0, st.A, st.A0, st.W2hat)
        assert np.isclose(drop - full, score[j], rtol=1e-9, atol=1e-9)


def test_brute_force_written_out_independently():
    """The enumerator itself, re-derived here directly from norms of the stacked residuals."""
    st = _tiny_state(3, d=4, f=7, T=15)
    k = 3
    Pi = np.linalg.pinv(st.X) @ st.X
    B = st.Z @ Pi
    best = None
    for keep in itertools.combinations(range(7), k):
        M = np.zeros(7)
        M[list(keep)] = 1
        val = np.sum((B - M[:, None] * st.Z0) ** 2)
        for j in range(7):
            val += np.sum(st.W2hat[:, j] ** 2) * np.sum((st.A0[j] - M[j] * st.A[j]) ** 2)
        if best is None or val < best[0]:
            best = (val, M)
    mask, val = orc.brute_force_mask(k, st.X, st.Z, st.Z0, st.A, st.A0, st.W2hat)
    assert np.array_equal(mask, best[1].astype(np.uint8))
    assert np.isclose(val, best[0], rtol=1e-10)


def test_wanda_rule_is_the_subset_optimum_of_the_output_term_at_init():
    st = _tiny_state(4, moved=False)
    k = 4
    bf_mask, _ = orc.brute_force_mask(k, st.X, st.Z, st.Z0, st.A, st.A0, st.W2hat, second_term_only=True)
    score = orc.module_scores(st, orc.WANDA)
    mask, _, _ = orc.select_topk(score, k)
    assert np.array_equal(mask, bf_mask)
    # WANDA score is the squared product of the column norm and the activation norm (eq. (wanda))
    ref = (np.linalg.norm(st.W2hat, axis=0) * np.linalg.norm(st.A, axis=1)) ** 2
    assert np.allclose(score, ref, rtol=1e-12)


def test_lemma_score_is_the_real_valued_minimiser_per_unit():
    st = _tiny_state(5)
    score = orc.module_scores(st, orc.LEMMA)
    Pi = np.linalg.pinv(st.X) @ st.X
    B = st.Z @ Pi
    for j in range(score.shape[0]):
        Dj = np.outer(st.W2hat[:, j], st.A[j])
        Yj = np.outer(st.W2hat[:, j], st.A0[j])
        fun = lambda m: np.sum((B[j] - m * st.Z0[j]) ** 2) + np.sum((Yj - m * Dj) ** 2)
        res = scipy.optimize.minimize_scalar(fun, bracket=(-2, 3), tol=1e-12)
        assert np.isclose(res.x, score[j], rtol=1e-6, atol=1e-8)


def test_lemma_ranking_is_not_the_binary_optimum_in_general_but_is_for_equal_denominators():
    # The printed s_j = P_j/Q_j ranks like the exact rule 2P_j - Q_j only when all Q_j agree.
    rng = np.random.default_rng(0)
    P = rng.normal(size=8) + 2
    Q = np.full(8, 3.0)
    lem = P / Q
    gain = 2 * P - Q
    assert np.array_equal(np.argsort(-lem, kind="stable"), np.argsort(-gain, kind="stable"))
    # unequal denominators: s = P/Q prefers unit 0 (0.9 > 0.75), the exact rule unit 1 (0.8 < 2.0)
    Q3 = np.array([1.0, 4.0])
    P3 = np.array([0.9, 3.0])
    assert np.argmax(P3 / Q3) == 0 and np.argmax(2 * P3 - Q3) == 1


def test_relaxed_lagrangian_stationary_point():
    st = _tiny_state(6)
    g, n2, e, u, v = orc.unit_sums(st.A, st.A0, st.Z, st.Z0, st.W2hat)
    P, Q = u + n2 * e, v + n2 * g
    n = P.shape[0]
    r = 0.4
    M, lam = orc.lemma_relaxed_mask(P, Q, r)
    assert np.isclose(np.sum(M), r * n, rtol=1e-12)
    # independent: minimise sum_j (Q_j M_j^2 - 2 P_j M_j) subject to sum M = r n (SLSQP)
    fun = lambda m: np.sum(Q * m * m - 2 * P * m)
    cons = {"type": "eq", "fun": lambda m: np.sum(m) - r * n}
    res = scipy.optimize.minimize(fun, np.full(n, r), constraints=[cons], method="SLSQP",
                                  options=dict(ftol=1e-14, maxiter=500))
    assert np.allclose(res.x, M, atol=1e-5)
    # lam = 0 gives r_l = mean_j s_j (eq. (rl))
    M0, lam0 = orc.lemma_relaxed_mask(P, Q, np.mean(P / Q))
    assert abs(lam0) < 1e-12 and np.allclose(M0, P / Q)


def test_scoring_identity_projection_form():
    """<C_j, B_j> with B = Z X^+ X equals sum_t Z0 Z (no pseudo-inverse needed for scoring)."""
    st = _tiny_state(7)
    Pi = np.linalg.pinv(st.X) @ st.X
    B = st.Z @ Pi
    _, _, _, u, v = orc.unit_sums(st.A, st.A0, st.Z, st.Z0, st.W2hat)
    assert np.allclose(np.einsum("jt,jt->j", B, st.Z0), u, rtol=1e-9)
    assert np.allclose(np.einsum("jt,jt->j", st.Z0, st.Z0), v)


def test_special_case_first_iteration_scores():
    st = _tiny_state(8, moved=False)
    g, n2, e, u, v = orc.unit_sums(st.A, st.A0, st.Z, st.Z0, st.W2hat)
    assert np.allclose(orc.unit_scores(g, n2, e, u, v, orc.LEMMA), 1.0, rtol=1e-12)
    assert np.allclose(orc.unit_scores(g, n2, e, u, v, orc.GAIN), v + n2 * g, rtol=1e-12)


def test_group_scores_sum_channels():
    st = _tiny_state(9, f=12)
    g, n2, e, u, v = orc.unit_sums(st.A, st.A0, st.Z, st.Z0, st.W2hat)
    s1 = orc.unit_scores(g, n2, e, u, v, orc.WANDA, group=1)
    s4 = orc.unit_scores(g, n2, e, u, v, orc.WANDA, group=4)
    assert np.allclose(s4, [s1[0:4].sum(), s1[4:8].sum(), s1[8:12].sum()])
    P, Q = u + n2 * e, v + n2 * g
    l4 = orc.unit_scores(g, n2, e, u, v, orc.LEMMA, group=4)
    assert np.allclose(l4, [P[i:i + 4].sum() / Q[i:i + 4].sum() for i in (0, 4, 8)])


# ---- P2: allocation ------------------------------------------------------------------
def test_allocation_sum_mean_and_counts():
    rng = np.random.default_rng(0)
    L = 12
    I = rng.uniform(0.5, 2.0, size=L)
    n = np.full(L, 3072)
    for rbar in (0.3, 0.5):
        for temp in (0.5, 1.0, 2.0, 10.0):
            r, npr = orc.softmax_allocation(I, n, rbar, temp)
            if not np.any(r == 0.95):
                assert np.isclose(np.sum(r), rbar * L, rtol=1e-12)
                assert np.isclose(np.mean(r), rbar, rtol=1e-12)
                assert np.sum(npr) == round(rbar * np.sum(n))
            assert np.all(r >= 0) and np.all(r <= 0.95)
            assert np.all(np.abs(npr - r * n) < 1.0 + 1e-9)
            # higher energy -> lower sparsity (monotone)
            order = np.argsort(I)
            assert np.all(np.diff(r[order]) <= 1e-15)


def test_allocation_closed_forms():
    # two layers: w_0 = sigmoid((I_1 - I_0)/(T * mean|I|))
    I = np.array([1.0, 3.0])
    temp = 0.7
    r, _ = orc.softmax_allocation(I, [100, 100], 0.4, temp)
    w0 = 1.0 / (1.0 + np.exp(-(3.0 - 1.0) / 2.0 / temp))
    assert np.allclose(r, [0.8 * w0, 0.8 * (1 - w0)], rtol=1e-12)
    # infinite temperature -> uniform ; equal energies -> uniform
    r, npr = orc.softmax_allocation(np.array([1.0, 2.0, 4.0]), [10, 10, 10], 0.5, 1e12)
    assert np.allclose(r, 0.5, atol=1e-9)
    r, npr = orc.softmax_allocation(np.array([2.0, 2.0, 2.0, 2.0]), [256] * 4, 0.5, 1.0)
    assert np.allclose(r, 0.5) and np.all(npr == 128)
    # smaller temperature concentrates the allocation
    I = np.array([1.0, 1.5, 2.0, 2.5])
    r_hot, _ = orc.softmax_allocation(I, [64] * 4, 0.3, 2.0)
    r_cold, _ = orc.softmax_allocation(I, [64] * 4, 0.3, 0.5)
    assert np.ptp(r_cold) > np.ptp(r_hot)


def test_allocation_clip_branch_and_groups():
    I = np.array([0.01, 5.0, 5.0, 5.0])
    r, npr = orc.softmax_allocation(I, [50] * 4, 0.5, 0.2)
    assert r[0] == 0.95 and np.all(r[1:] < 0.5)       # clipped layer, no rescale afterwards
    assert npr[0] == round(0.95 * 50) or npr[0] == int(0.95 * 50)
    # two softmax groups are allocated independently
    I = np.array([1.0, 2.0, 1.0, 2.0])
    r, _ = orc.softmax_allocation(I, [64] * 4, 0.5, 1.0, group_id=[0, 0, 1, 1])
    assert np.allclose(r[:2], r[2:]) and np.isclose(r[:2].mean(), 0.5)
    # at least one unit survives per layer
    r, npr = orc.softmax_allocation(np.array([1.0]), [4], 0.95, 1.0)
    assert npr[0] <= 3


# ---- O4 select ---------------------------------------------------------------------
def test_select_topk_ties_and_threshold():
    score = np.array([3.0, 1.0, 3.0, 2.0, 3.0, 0.5])
    mask, idx, tau = orc.select_topk(score, 2)
    assert idx.tolist() == [0, 2] and tau == 3.0 and mask.tolist() == [1, 0, 1, 0, 0, 0]
    mask, idx, tau = orc.select_topk(score, 4)
    assert idx.tolist() == [0, 2, 3, 4] and tau == 2.0
    mask, idx, tau = orc.select_topk(np.array([5.0, 1.0, 7.0]), 2, group=2)
    assert idx.tolist() == [0, 1, 4, 5]


# ---- P3: Gram ------------------------------------------------------------------------
def test_gram_properties():
    rng = np.random.default_rng(1)
    A = rng.normal(size=(7, 33))
    idx = np.array([1, 3, 6])
    G = orc.gram(A, idx)
    assert np.allclose(G, G.T)
    assert np.allclose(np.diag(G), np.sum(A[idx] ** 2, axis=1))
    assert np.all(np.linalg.eigvalsh(G) > -1e-10)
    ref = np.array([[np.dot(A[i], A[j]) for j in idx] for i in idx])
    assert np.allclose(G, ref)


# ---- P4: refits ----------------------------------------------------------------------
def test_refit_normal_equations_and_lstsq_limit():
    st = _tiny_state(10, d=6, f=10, T=60)
    idx = np.array([0, 2, 3, 7, 9])
    d, f = 6, 10
    W2 = orc.refit_fc2(st.Y, st.A, idx, st.lam2, d, f)
    G = st.A[idx] @ st.A[idx].T
    R2 = st.Y @ st.A[idx].T
    assert np.linalg.norm(W2[:, idx] @ (G + st.lam2 * np.eye(5)) - R2) / np.linalg.norm(R2) < 1e-10
    assert np.all(W2[:, [1, 4, 5, 6, 8]] == 0)
    W1 = orc.refit_fc1(st.Z, st.X, idx, st.H, st.lam1, d, f)
    R1 = st.Z[idx] @ st.X.T
    assert np.linalg.norm(W1[idx] @ (st.H + st.lam1 * np.eye(d)) - R1) / np.linalg.norm(R1) < 1e-10
    assert np.all(W1[[1, 4, 5, 6, 8]] == 0)
    # lam -> 0: plain least squares via the library routine
    W2z = orc.refit_fc2(st.Y, st.A, idx, 0.0, d, f)
    ls = np.linalg.lstsq(st.A[idx].T, st.Y.T, rcond=None)[0].T
    assert np.allclose(W2z[:, idx], ls, rtol=1e-8, atol=1e-10)
    W1z = orc.refit_fc1(st.Z, st.X, idx, st.H, 0.0, d, f)
    ls1 = np.linalg.lstsq(st.X.T, st.Z[idx].T, rcond=None)[0].T
    assert np.allclose(W1z[idx], ls1, rtol=1e-8, atol=1e-10)
    # ridge: equals least squares on the system augmented with sqrt(lam) I
    aug_A = np.hstack([st.A[idx], np.sqrt(st.lam2) * np.eye(5)])
    aug_Y = np.hstack([st.Y, np.zeros((d, 5))])
    ls2 = np.linalg.lstsq(aug_A.T, aug_Y.T, rcond=None)[0].T
    assert np.allclose(W2[:, idx], ls2, rtol=1e-8, atol=1e-10)


def test_fc1_restrict_then_fit_equals_fit_then_restrict_at_init():
    st = _tiny_state(11, moved=False, d=6, f=10, T=60)
    idx = np.array([1, 2, 5])
    W1 = orc.refit_fc1(st.Z, st.X, idx, st.H, 0.0, 6, 10)
    assert np.allclose(W1[idx], st.W1hat[idx], rtol=1e-8, atol=1e-10)


# ---- P5: a-update --------------------------------------------------------------------
def test_a_update_is_the_ridge_solution():
    st = _tiny_state(12, d=6, f=10, T=40)
    idx = np.array([0, 2, 3, 7, 9])
    alpha, beta = 0.7, 1.3
    W2 = orc.refit_fc2(st.Y, st.A, idx, st.lam2, 6, 10)
    A = orc.a_update(W2, st.Y, st.Z, alpha, beta)
    # stacked least squares with the library routine
    lhs = np.vstack([np.sqrt(alpha) * W2, np.sqrt(beta) * np.eye(10)])
    rhs = np.vstack([np.sqrt(alpha) * st.Y, np.sqrt(beta) * np.maximum(st.Z, 0)])
    ref = np.linalg.lstsq(lhs, rhs, rcond=None)[0]
    assert np.allclose(A, ref, rtol=1e-9, atol=1e-11)
    # pruned rows decouple
    off = np.setdiff1d(np.arange(10), idx)
    assert np.allclose(A[off], np.maximum(st.Z[off], 0))
    # Woodbury / residual form on the kept rows
    W = W2[:, idx]
    Mm = (beta / alpha) * np.eye(6) + W @ W.T
    E = st.Y - W @ np.maximum(st.Z[idx], 0)
    assert np.allclose(A[idx], np.maximum(st.Z[idx], 0) + W.T @ np.linalg.solve(Mm, E), rtol=1e-9, atol=1e-11)
    # gradient of the block objective vanishes
    grad = -2 * alpha * W2.T @ (st.Y - W2 @ A) + 2 * beta * (A - np.maximum(st.Z, 0))
    assert np.max(np.abs(grad)) < 1e-9


def test_output_residual_after_the_a_update_is_a_scaled_solve_of_the_old_residual():
    """After the a-update, Y - W2 A = (beta/alpha) M^-1 E with E the residual before it, so the first objective term
    is (beta/alpha)^2 <M^-2, E E^T> (what the GPU path reports after an a-update); false for any other A."""
    st = _tiny_state(21, d=6, f=10, T=40)
    idx = np.array([1, 2, 4, 7, 8])
    alpha, beta = 0.7, 1.3
    W2 = orc.refit_fc2(st.Y, st.A, idx, st.lam2, 6, 10)
    A = orc.a_update(W2, st.Y, st.Z, alpha, beta)
    W = W2[:, idx]
    c = beta / alpha
    Mm = c * np.eye(6) + W @ W.T
    E = st.Y - W @ np.maximum(st.Z[idx], 0)
    res = st.Y - W2 @ A
    assert np.allclose(res, c * np.linalg.solve(Mm, E), rtol=1e-9, atol=1e-11)
    Minv = np.linalg.inv(Mm)
    assert np.isclose(np.sum(res * res), c * c * np.sum((Minv @ Minv) * (E @ E.T)), rtol=1e-10)
    A_other = A + 1e-3
    assert not np.isclose(np.sum((st.Y - W2 @ A_other) ** 2), c * c * np.sum((Minv @ Minv) * (E @ E.T)), rtol=1e-6)


# ---- P6: z-update --------------------------------------------------------------------
def test_z_update_beats_grid_search():
    st = _tiny_state(13, d=4, f=6, T=10)
    alpha, beta = 0.8, 1.1
    Z = orc.z_update(st.W1, st.X, st.A, alpha, beta)
    Z1 = st.W1 @ st.X
    grid = np.linspace(-8, 8, 32001)
    for j in range(6):
        for t in range(10):
            cost = beta * (st.A[j, t] - np.maximum(grid, 0)) ** 2 + alpha * (grid - Z1[j, t]) ** 2
            c_closed = beta * (st.A[j, t] - max(Z[j, t], 0)) ** 2 + alpha * (Z[j, t] - Z1[j, t]) ** 2
            assert c_closed <= cost.min() + 1e-12
            assert abs(grid[np.argmin(cost)] - Z[j, t]) < 1e-3 or abs(cost.min() - c_closed) < 1e-6


# ---- P7: monotone objective on config 1 -------------------------------------------------
def test_admm_objective_non_increasing_config1(tiny_np):
    cfg, m = tiny_np
    st = orc.module_init(m["W1hat"], m["W2hat"], m["X"], delta=0.01)
    k = cfg.f - int(round(cfg.rbar * cfg.f))
    prev = None
    for it in range(cfg.K):
        trace = []
        orc.admm_step(st, k, 1.0, 1.0, orc.WANDA, select=(it == 0), trace=trace)
        if it > 0:
            seq = [prev] + trace
            for a, b in zip(seq[:-1], seq[1:]):
                assert b <= a * (1 + 1e-10) + 1e-12
        else:
            # a- and z-updates are exact minimisers even when the mask has just changed
            assert trace[2] <= trace[1] * (1 + 1e-10) and trace[3] <= trace[2] * (1 + 1e-10)
        prev = trace[-1]
    assert st.history[-1].sum() < st.history[0].sum()
    assert int(st.mask.sum()) == k


def test_reselect_mode_runs_and_counts(tiny_np):
    cfg, m = tiny_np
    st = orc.module_init(m["W1hat"], m["W2hat"], m["X"])
    for it in range(3):
        orc.admm_step(st, 100, 1.0, 1.0, orc.GAIN, select=True)
        assert int(st.mask.sum()) == 100 and st.idx.shape[0] == 100
        assert np.all(st.W2[:, st.mask == 0] == 0) and np.all(st.W1[st.mask == 0] == 0)


# ---- P9 + driver -----------------------------------------------------------------------
def test_driver_temperature_sweep_small():
    rng = np.random.default_rng(3)
    mods = []
    for l in range(3):
        X = rng.normal(size=(8, 64)) * (1 + 0.2 * l)
        mods.append((rng.normal(size=(16, 8)) * 0.3, rng.normal(size=(8, 16)) * 0.3, X))
    res, best = orc.prune_model(mods, 0.5, [0.5, 2.0], K=3)
    assert best in (0.5, 2.0)
    assert res[best]["total"] == min(r["total"] for r in res.values())
    for r in res.values():
        assert int(np.sum(r["nprune"])) == 24
        # layers with larger energy are pruned less
        o = np.argsort(r["energies"])
        assert np.all(np.diff(r["r"][o]) <= 1e-15)


def test_head_variant_refit():
    rng = np.random.default_rng(5)
    d, g, T = 12, 3, 80
    WO = rng.normal(size=(d, d)) * 0.2
    C = rng.normal(size=(d, T)) * rng.uniform(0.2, 2.0, size=(d, 1))
    out = orc.head_prune(WO, C, g, 2)
    assert out["idx"].shape[0] == 6 and out["mask"].sum() == 2
    idx = out["idx"]
    G = C[idx] @ C[idx].T
    R = out["Y"] @ C[idx].T
    res = out["WO"][:, idx] @ (G + out["lam"] * np.eye(6)) - R
    assert np.linalg.norm(res) / np.linalg.norm(R) < 1e-10
    # head scores by enumeration of what dropping a head costs in the output term at init
    for h in range(4):
        ch = np.arange(h * g, (h + 1) * g)
        cost = sum(np.sum(np.outer(WO[:, j], C[j]) ** 2) for j in ch)
        assert np.isclose(cost, out["score"][h])


# ---- shapes of the workloads (Tables 1 and 2) --------------------------------------------
def test_config_shapes_match_tables():
    from paper_2510_03246_amd import inputs
    ffn_params = {"opt125m": 4_718_592, "opt1.3b": 33_554_432, "opt6.7b": 134_217_728, "opt30b": 411_041_792}
    layers = {"opt125m": 12, "opt1.3b": 24, "opt6.7b": 32, "opt30b": 48}
    for name, p in ffn_params.items():
        c = inputs.CONFIGS[name]
        assert 2 * c.d * c.f == p == 8 * c.d * c.d
        assert c.L == layers[name]


# ---------------------------------------------------------------------------------------------
# Alg. 2: weight-only importances and inverse weighting
# ---------------------------------------------------------------------------------------------
def test_weight_importance_hand_values():
    """A 2 x 2 matrix worked by hand: |W|_1 = 10, mean = -0.5, Var = 30/4 - 0.25 = 7.25, |W|_2 = sqrt(30)."""
    W = np.array([[1.0, -2.0], [3.0, -4.0]])
    assert orc.weight_importance([W], 0.0) == 10.0
    assert np.isclose(orc.weight_importance([W], 1.0) - 10.0, 7.25, rtol=1e-14)
    assert np.isclose(orc.weight_importance([W], 0.0, 1.0) - 10.0, np.sqrt(30.0), rtol=1e-14)
    # a group of two slices pools its entries: same numbers from the two rows given separately
    assert np.isclose(orc.weight_importance([W[0], W[1]], 0.1, 0.01, 2.0), 2.0 * (10.0 + 0.725 + 0.01 * np.sqrt(30.0)), rtol=1e-14)
    # the layer formula: MLP = fc1 and fc2 scored separately, depth decay gamma^l
    I = orc.layer_importance_alg2("mlp", 3, [[W], [2 * W]], gamma=0.5)
    assert np.isclose(I, 0.125 * ((10.0 + 0.05 * 7.25) + (20.0 + 0.05 * 29.0)), rtol=1e-14)
    Ia = orc.layer_importance_alg2("attn", 1, [[W], [W]], gamma=0.9, rho=2.0)
    assert np.isclose(Ia, 0.9 * 2.0 * 2 * (10.0 + 0.725 + 0.01 * np.sqrt(30.0)), rtol=1e-14)


def test_inverse_allocation_identities():
    rng = np.random.default_rng(3)
    L = 12
    I = rng.uniform(1.0, 3.0, size=L)
    n = np.full(L, 1000)
    r, npr = orc.inverse_allocation(I, n, 0.5, 1.0)
    assert np.isclose(np.sum(r), 0.5 * L, rtol=1e-12)            # nothing clipped: the mean is rbar
    assert np.sum(npr) == int(np.rint(np.sum(r * n)))
    # as printed: w = softmax(-I/T) falls with I, so 1 - w and the sparsity RISE with the importance
    order = np.argsort(I)
    assert np.all(np.diff(r[order]) >= 0)
    # T -> infinity: uniform
    r_inf, _ = orc.inverse_allocation(I, n, 0.5, 1e9)
    assert np.allclose(r_inf, 0.5, rtol=1e-6)
    # two layers, closed form: scaled energies a, b with mean 1; w1 = 1 / (1 + exp((a - b)/T)); r1 = 2 rbar (1 - w1)
    a, b = 0.8, 1.2
    r2, _ = orc.inverse_allocation(np.array([a, b]) * 7.0, np.array([10, 10]), 0.4, 0.5)
    w1 = 1.0 / (1.0 + np.exp((a - b) / 0.5))
    assert np.allclose(r2, [0.8 * (1 - w1), 0.8 * w1], rtol=1e-12)
    # one layer per group: r = rbar; the clip binds at rmax
    r1, _ = orc.inverse_allocation(np.array([5.0, 1.0, 2.0]), np.array([8, 8, 8]), 0.3, 1.0, group_id=np.array([0, 1, 1]))
    assert r1[0] == 0.3
    rc, _ = orc.inverse_allocation(np.array([1.0, 50.0]), np.array([100, 100]), 0.9, 0.05)
    assert np.max(rc) == 0.95 and np.min(rc) >= 0.0


# ---- hand-worked 2 x 2 module: initialisation constants and every term of the objective ------------
def _hand_module():
    W1hat = np.array([[1.0, -1.0], [2.0, 0.0]])
    W2hat = np.array([[1.0, 0.0], [0.5, -1.0]])
    X = np.array([[1.0, 2.0], [3.0, -1.0]])
    return orc.module_init(W1hat, W2hat, X, delta=0.1)


def test_module_init_hand_values():
    """Z0 = W1hat X = [[-2, 3], [2, 4]]; A0 = ReLU; Y = W2hat A0 = [[0, 3], [-2, -2.5]]; H = X X^T = [[5, 1], [1, 10]];
    lam1 = delta tr(H) / d = 0.1 * 15 / 2; lam2 = delta |A0|_F^2 / f = 0.1 * (9 + 4 + 16) / 2 (worked by hand)."""
    st = _hand_module()
    assert np.array_equal(st.Z0, [[-2.0, 3.0], [2.0, 4.0]])
    assert np.array_equal(st.A0, [[0.0, 3.0], [2.0, 4.0]])
    assert np.array_equal(st.Y, [[0.0, 3.0], [-2.0, -2.5]])
    assert np.array_equal(st.H, [[5.0, 1.0], [1.0, 10.0]])
    assert st.lam1 == pytest.approx(0.75, rel=1e-15)
    assert st.lam2 == pytest.approx(1.45, rel=1e-15)
    assert np.array_equal(st.Z, st.Z0) and np.array_equal(st.A, st.A0)


def test_objective_terms_hand_values():
    """alpha = 2, beta = 3, T = 2 on a state written by hand (unit 1 pruned):
       Y - W2 A = [[-0.5, 1], [-2, -2.5]]  -> 11.5;   A - ReLU(Z) = [[0.5, 0], [0, 0]] -> 0.25;
       Z - W1 X = [[-2, 0], [1, 3]] -> 14;  |W2|^2 = |W1|^2 = 1;  lam2 = 1.45, lam1 = 0.75.
       terms = [2 * 11.5, 3 * 0.25, 2 * 14, 2 * 1.45 * 1, 2 * 0.75 * 1] / 2."""
    st = _hand_module()
    st.Z = np.array([[-1.0, 2.0], [1.0, 3.0]])
    st.A = np.array([[0.5, 2.0], [1.0, 3.0]])
    st.W1 = np.array([[1.0, 0.0], [0.0, 0.0]])
    st.W2 = np.array([[1.0, 0.0], [0.0, 0.0]])
    terms = orc.objective_terms(st, 2.0, 3.0)
    assert np.allclose(terms, [11.5, 0.375, 14.0, 1.45, 0.75], rtol=1e-14, atol=0)
    assert orc.objective(st, 2.0, 3.0) == pytest.approx(28.075, rel=1e-14)
    assert orc.objective(st, 2.0, 3.0, ridge=False) == pytest.approx(25.875, rel=1e-14)
