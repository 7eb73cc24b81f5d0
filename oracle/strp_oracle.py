"""Plain fp64 numpy oracle of the per-module ADMM structured-pruning subproblem.

TEST INFRASTRUCTURE ONLY -- never imported by the product path, shares nothing with the
HIP library.  Every function restates one passage of the paper (cited per function) in the
paper's order and notation, with no blocking, fusion or reordering.

Orientation (row-major, tokens are the trailing axis):
    X   [d, T]  input of fc1  (a^pre_{l-1})          W1hat [f, d]  fc1 (\\hat W_l)
    Z   [f, T]  pre-activation auxiliary  (z_l)      W2hat [d, f]  fc2 (\\hat W_{l+1})
    A   [f, T]  post-activation auxiliary (a_l)      Y     [d, T]  module output target (z^pre_{l+1})
A structured unit j of an FFN module is hidden neuron j: row j of W1 and column j of W2.

Readings taken where the paper is silent or inconsistent (each also listed in the design
notes of the repository):
  * every per-unit product in Lemma 1 is a sum over the T calibration tokens;
  * the second Lemma-1 term is made separable over hidden units by comparing unit j's
    rank-one contribution D_j = W2hat[:, j] A_j with the dense model's own contribution
    Y_j = W2hat[:, j] A0_j  (so sum_j Y_j = Y);
  * <C_j, B_j> = <Z0_j, Z_j> because Z0_j already lies in the row space of X;
  * r_l is the pruned fraction (Alg. 1), exactly k = n - nprune units are kept;
  * weights are recovered by ridge least squares restricted to the kept support, the
    damping lam = delta * mean(diag Gram) fixed at initialisation;
  * the z rule is the exact per-element minimiser of the two-term z subproblem.
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass, field

import numpy as np

WANDA, LEMMA, GAIN = 0, 1, 2


# --------------------------------------------------------------------------------------
# O0  initialisation (Alg. 3, "Initialize z = z^pre, a = a^pre", cached input Gram)
# --------------------------------------------------------------------------------------
@dataclass
class ModuleState:
    X: np.ndarray
    W1hat: np.ndarray
    W2hat: np.ndarray
    Z0: np.ndarray
    A0: np.ndarray
    Y: np.ndarray
    H: np.ndarray
    lam1: float
    lam2: float
    Z: np.ndarray
    A: np.ndarray
    W1: np.ndarray
    W2: np.ndarray
    mask: np.ndarray | None = None
    idx: np.ndarray | None = None
    history: list = field(default_factory=list)


def module_init(W1hat, W2hat, X, delta=0.01) -> ModuleState:
    """Dense forward of the module on the calibration tokens and the fixed ridge dampings.

    Alg. 3 (FFN function): z <- z^pre, a <- a^pre; the cached pseudo-inverse of the input
    is represented by the input Gram H = X X^T.  phi is ReLU (Appendix A.1).  No biases.
    """
    W1hat = np.asarray(W1hat, dtype=np.float64)
    W2hat = np.asarray(W2hat, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    f, d = W1hat.shape
    Z0 = W1hat @ X
    A0 = np.maximum(Z0, 0.0)
    Y = W2hat @ A0
    H = X @ X.T
    lam1 = delta * np.trace(H) / d
    lam2 = delta * np.sum(A0 * A0) / f
    return ModuleState(X=X, W1hat=W1hat, W2hat=W2hat, Z0=Z0, A0=A0, Y=Y, H=H,
                       lam1=float(lam1), lam2=float(lam2), Z=Z0.copy(), A=A0.copy(),
                       W1=W1hat.copy(), W2=W2hat.copy())


# --------------------------------------------------------------------------------------
# O1/O2  per-unit sums and structural scores (Lemma 1; eq. (wanda))
# --------------------------------------------------------------------------------------
def unit_sums(A, A0, Z, Z0, W2hat):
    """Token sums every score mode is built from.

    g_j = sum_t A_jt^2,  n2_j = sum_i W2hat[i,j]^2,  e_j = sum_t A_jt A0_jt,
    u_j = sum_t Z0_jt Z_jt,  v_j = sum_t Z0_jt^2.
    With b, c, d of Lemma 1 summed over tokens:  c.b = u, c.c = v, |d|^2 = n2*g, d.y = n2*e.
    """
    g = np.einsum("jt,jt->j", A, A)
    n2 = np.einsum("ij,ij->j", W2hat, W2hat)
    e = np.einsum("jt,jt->j", A, A0)
    u = np.einsum("jt,jt->j", Z0, Z)
    v = np.einsum("jt,jt->j", Z0, Z0)
    return g, n2, e, u, v


def unit_scores(g, n2, e, u, v, mode, group=1):
    """Structural score per unit (a unit is `group` consecutive channels; heads use group=d_head).

    WANDA: (|W2hat[:,j]|_2 * |A_j|_2)^2 = n2_j g_j   (square of eq. (wanda): same ranking)
    LEMMA: s_j = (c_j b_j + d_j z_j) / (c_j^2 + d_j^2) = P_j / Q_j      (Lemma 1)
    GAIN : Phi(M_j = 0) - Phi(M_j = 1) = 2 P_j - Q_j   (exact binary rule for eq. (78))
    """
    P = u + n2 * e
    Q = v + n2 * g
    n = g.shape[0] // group

    def gsum(x):
        return x.reshape(n, group).sum(axis=1)

    if mode == WANDA:
        return gsum(n2 * g)
    if mode == LEMMA:
        return gsum(P) / gsum(Q)
    if mode == GAIN:
        return gsum(2.0 * P - Q)
    raise ValueError("unknown score mode")


def layer_energy(score):
    """I_l: the layer importance is the mean unit score (eq. (rl) / proof, with j over units)."""
    return float(np.mean(score))


def lemma_relaxed_mask(P, Q, r_keep):
    """Stationary point of the relaxed per-layer Lagrangian (eqs. (opti), (lambdas), (Mlj)).

    Returns (M, lam) with M_j = (P_j - lam/2)/Q_j and sum_j M_j = r_keep * n.
    """
    n = P.shape[0]
    lam = 2.0 * (np.sum(P / Q) - r_keep * n) / np.sum(1.0 / Q)
    return (P - 0.5 * lam) / Q, lam


# --------------------------------------------------------------------------------------
# O3  softmax sparsity allocation (Lemma 2; Alg. 1 steps 1-2)
# --------------------------------------------------------------------------------------
def softmax_allocation(I, n_units, rbar, temperature, rmax=0.95, group_id=None):
    """Per-layer pruned fractions r_l and integer prune counts.

    Per softmax group (e.g. all FFN modules): energies are scaled by the group's mean |I|
    so the temperature is scale-free, w = softmax(-I/T), r = rbar * L * w, clip to
    [0, rmax]; if no entry sits at rmax: rescale by rbar/mean(r) and clip again.
    Integer counts: largest-remainder rounding of r_l * n_l per group so that the total
    equals round(sum r_l n_l); every layer keeps at least one unit.
    """
    I = np.asarray(I, dtype=np.float64)
    n_units = np.asarray(n_units, dtype=np.int64)
    L = I.shape[0]
    if group_id is None:
        group_id = np.zeros(L, dtype=np.int64)
    group_id = np.asarray(group_id)
    r = np.zeros(L)
    nprune = np.zeros(L, dtype=np.int64)
    for gid in np.unique(group_id):
        sel = np.nonzero(group_id == gid)[0]
        Lg = sel.shape[0]
        Ig = I[sel]
        scale = np.mean(np.abs(Ig))
        In = Ig / scale if scale > 0 else np.zeros(Lg)
        a = -In / temperature
        a = a - np.max(a)
        w = np.exp(a)
        w = w / np.sum(w)
        rg = rbar * Lg * w
        rg = np.minimum(np.maximum(rg, 0.0), rmax)
        if not np.any(rg == rmax):
            mu = np.mean(rg)
            rg = rg * (rbar / mu)
            rg = np.minimum(np.maximum(rg, 0.0), rmax)
        r[sel] = rg
        x = rg * n_units[sel]
        base = np.floor(x).astype(np.int64)
        extra = int(np.rint(np.sum(x))) - int(np.sum(base))
        frac = x - base
        order = np.argsort(-frac, kind="stable")
        for t in range(max(extra, 0)):
            base[order[t % Lg]] += 1
        base = np.minimum(base, n_units[sel] - 1)
        base = np.maximum(base, 0)
        nprune[sel] = base
    return r, nprune


# --------------------------------------------------------------------------------------
# Alg. 2: weight-only layer importances and temperature-guided inverse weighting
# --------------------------------------------------------------------------------------
def weight_importance(mats, var_coef, l2_coef=0.0, scale=1.0):
    """scale * (|W|_1 + var_coef * Var(W) + l2_coef * |W|_2) of ONE parameter group (Alg. 2 step 1).

    `mats` is a list of arrays that together form the group (a head's slices of the four
    attention matrices, or a single fc matrix): the 1-norm is the sum of absolute values,
    Var the population variance over every entry of the group, |.|_2 the Euclidean
    (Frobenius) norm of the entries.
    """
    v = np.concatenate([np.asarray(m, dtype=np.float64).ravel() for m in mats])
    l1 = np.sum(np.abs(v))
    var = np.mean(v * v) - np.mean(v) ** 2
    l2 = np.sqrt(np.sum(v * v))
    return float(scale * (l1 + var_coef * var + l2_coef * l2))


def layer_importance_alg2(kind, layer, groups, gamma, rho=1.0):
    """I_l of Alg. 2: depth decay gamma^l (l counted from 1) times, for an attention layer,
    rho * sum over heads of (|W_h|_1 + 0.1 Var(W_h) + 0.01 |W_h|_2); for an MLP layer,
    sum over fc1, fc2 of (|W_m|_1 + 0.05 Var(W_m)).  `groups` = list of parameter groups
    (each a list of arrays): the heads, or [[fc1], [fc2]]."""
    d = gamma ** layer
    if kind == "attn":
        return sum(weight_importance(g, 0.1, 0.01, d * rho) for g in groups)
    if kind == "mlp":
        return sum(weight_importance(g, 0.05, 0.0, d) for g in groups)
    raise ValueError(kind)


def inverse_allocation(I, n_units, rbar, temperature, rmax=0.95, group_id=None):
    """Alg. 2 step 2: per group w = softmax(-I/T) (energies scaled by the group's mean |I|, as in
    softmax_allocation), r = clip(rbar * L * (1 - w) / sum(1 - w), 0, rmax).  No rescale step.
    A group with a single layer gets r = rbar (1 - w = 0 there).  Integer counts as in
    softmax_allocation."""
    I = np.asarray(I, dtype=np.float64)
    n_units = np.asarray(n_units, dtype=np.int64)
    L = I.shape[0]
    if group_id is None:
        group_id = np.zeros(L, dtype=np.int64)
    group_id = np.asarray(group_id)
    r = np.zeros(L)
    nprune = np.zeros(L, dtype=np.int64)
    for gid in np.unique(group_id):
        sel = np.nonzero(group_id == gid)[0]
        Lg = sel.shape[0]
        Ig = I[sel]
        scale = np.mean(np.abs(Ig))
        In = Ig / scale if scale > 0 else np.zeros(Lg)
        a = -In / temperature
        a = a - np.max(a)
        w = np.exp(a)
        w = w / np.sum(w)
        if Lg > 1:
            rg = rbar * Lg * (1.0 - w) / np.sum(1.0 - w)
        else:
            rg = np.full(1, rbar)
        rg = np.minimum(np.maximum(rg, 0.0), rmax)
        r[sel] = rg
        x = rg * n_units[sel]
        base = np.floor(x).astype(np.int64)
        extra = int(np.rint(np.sum(x))) - int(np.sum(base))
        frac = x - base
        order = np.argsort(-frac, kind="stable")
        for t in range(max(extra, 0)):
            base[order[t % Lg]] += 1
        base = np.minimum(base, n_units[sel] - 1)
        base = np.maximum(base, 0)
        nprune[sel] = base
    return r, nprune


# --------------------------------------------------------------------------------------
# O4  top-k structured mask (threshold rule below Lemma 1; Alg. 4 threshold step)
# --------------------------------------------------------------------------------------
def select_topk(score, k, group=1):
    """Keep exactly the k highest-scoring units; equal scores keep the lower index.

    Returns (unit mask [n] uint8, kept channel indices ascending [k*group], tau = lowest kept score).
    """
    score = np.asarray(score)
    n = score.shape[0]
    order = np.argsort(-score, kind="stable")
    kept = np.sort(order[:k])
    mask = np.zeros(n, dtype=np.uint8)
    mask[kept] = 1
    tau = float(np.min(score[kept])) if k > 0 else float("inf")
    idx = (kept[:, None] * group + np.arange(group)[None, :]).reshape(-1)
    return mask, idx.astype(np.int64), tau


# --------------------------------------------------------------------------------------
# O5/O6  restricted ridge least squares ("reversely recovering the weight matrix", W = z a^+)
# --------------------------------------------------------------------------------------
def gram(A, idx=None):
    """G = A_S A_S^T over the tokens."""
    As = A if idx is None else A[idx]
    return As @ As.T


def refit_fc2(Y, A, idx, lam2, d, f):
    """W2[:, S] = argmin_W |Y - W A_S|^2 + lam2 |W|^2 ; other columns zero."""
    As = A[idx]
    G = As @ As.T
    R2 = Y @ As.T
    Ws = np.linalg.solve(G + lam2 * np.eye(G.shape[0]), R2.T).T
    W2 = np.zeros((d, f))
    W2[:, idx] = Ws
    return W2


def refit_fc1(Z, X, idx, H, lam1, d, f):
    """W1[S, :] = argmin_W |Z_S - W X|^2 + lam1 |W|^2 ; other rows zero."""
    R1 = Z[idx] @ X.T
    Ws = np.linalg.solve(H + lam1 * np.eye(d), R1.T).T
    W1 = np.zeros((f, d))
    W1[idx, :] = Ws
    return W1


# --------------------------------------------------------------------------------------
# O7  a-update (Appendix A.1 "Updating activation")
# --------------------------------------------------------------------------------------
def a_update(W2, Y, Z, alpha, beta):
    """a = (alpha W2^T W2 + beta I)^-1 (alpha W2^T Y + beta ReLU(Z)), full f x f system."""
    f = W2.shape[1]
    lhs = alpha * (W2.T @ W2) + beta * np.eye(f)
    rhs = alpha * (W2.T @ Y) + beta * np.maximum(Z, 0.0)
    return np.linalg.solve(lhs, rhs)


# --------------------------------------------------------------------------------------
# O8  z-update (Appendix A.1 "Updating output")
# --------------------------------------------------------------------------------------
def z_update(W1, X, A, alpha, beta, rule="exact", Z_old=None):
    """Per-element minimiser of beta (a - ReLU(z))^2 + alpha (z - z1)^2 with z1 = W1 X.

    On z <= 0 the cost is beta a^2 + alpha (z - z1)^2, minimised at min(z1, 0);
    on z >= 0 it is beta (a - z)^2 + alpha (z - z1)^2, minimised at max(z2, 0) with
    z2 = (beta a + alpha z1)/(alpha + beta).  Keep the cheaper; a tie keeps the z >= 0 branch.
    rule="paper_sign" is the literal listing (sign test on the previous z), for comparison only.
    """
    Z1 = W1 @ X
    Z2 = (beta * A + alpha * Z1) / (alpha + beta)
    if rule == "paper_sign":
        return np.where(Z_old < 0, Z1, Z2)
    cm = np.minimum(Z1, 0.0)
    cost_m = beta * A * A + alpha * (cm - Z1) ** 2
    cp = np.maximum(Z2, 0.0)
    cost_p = beta * (A - cp) ** 2 + alpha * (cp - Z1) ** 2
    return np.where(cost_m < cost_p, cm, cp)


# --------------------------------------------------------------------------------------
# O9  objective (FFN objective of Appendix A.1, per token)
# --------------------------------------------------------------------------------------
def objective_terms(st: ModuleState, alpha, beta):
    """(1/T) [ alpha|Y - W2 A|^2, beta|A - ReLU(Z)|^2, alpha|Z - W1 X|^2, alpha lam2|W2|^2, alpha lam1|W1|^2 ]."""
    T = st.X.shape[1]
    t1 = alpha * np.sum((st.Y - st.W2 @ st.A) ** 2)
    t2 = beta * np.sum((st.A - np.maximum(st.Z, 0.0)) ** 2)
    t3 = alpha * np.sum((st.Z - st.W1 @ st.X) ** 2)
    t4 = alpha * st.lam2 * np.sum(st.W2 ** 2)
    t5 = alpha * st.lam1 * np.sum(st.W1 ** 2)
    return np.array([t1, t2, t3, t4, t5]) / T


def objective(st: ModuleState, alpha, beta, ridge=True):
    t = objective_terms(st, alpha, beta)
    return float(np.sum(t) if ridge else np.sum(t[:3]))


# --------------------------------------------------------------------------------------
# One inner iteration (Alg. 3 FFN loop body / Alg. 4 step body)
# --------------------------------------------------------------------------------------
def module_scores(st: ModuleState, mode, group=1):
    g, n2, e, u, v = unit_sums(st.A, st.A0, st.Z, st.Z0, st.W2hat)
    return unit_scores(g, n2, e, u, v, mode, group)


def admm_step(st: ModuleState, k, alpha=1.0, beta=1.0, mode=WANDA, select=True, trace=None):
    """score -> top-k -> refit fc2 -> refit fc1 -> a-update -> z-update -> objective.

    `select=False` keeps the mask of the previous iteration (Alg. 1 ordering: the mask is
    chosen once, then the ADMM loop runs).  The score always uses the original W2hat.
    `trace`, if a list, receives the objective after each of the four block updates.
    """
    f, d = st.W1hat.shape
    if select or st.idx is None:
        score = module_scores(st, mode)
        st.mask, st.idx, tau = select_topk(score, k)
        st.score, st.tau = score, tau
    idx = st.idx
    st.W2 = refit_fc2(st.Y, st.A, idx, st.lam2, d, f)
    if trace is not None:
        trace.append(objective(st, alpha, beta))
    st.W1 = refit_fc1(st.Z, st.X, idx, st.H, st.lam1, d, f)
    if trace is not None:
        trace.append(objective(st, alpha, beta))
    st.A = a_update(st.W2, st.Y, st.Z, alpha, beta)
    if trace is not None:
        trace.append(objective(st, alpha, beta))
    st.Z = z_update(st.W1, st.X, st.A, alpha, beta)
    terms = objective_terms(st, alpha, beta)
    if trace is not None:
        trace.append(float(np.sum(terms)))
    st.history.append(terms)
    return terms


# --------------------------------------------------------------------------------------
# Head variant: output projection of an attention module, units = heads of g channels
# --------------------------------------------------------------------------------------
def head_prune(WOhat, C, g, k_heads, delta=0.01):
    """Score heads by the grouped WANDA score, keep k_heads, ridge-refit W_O on the kept channels.

    C [d, T] is the concatenated head output, Y = WOhat C the projection's dense output.
    """
    WOhat = np.asarray(WOhat, dtype=np.float64)
    C = np.asarray(C, dtype=np.float64)
    d = WOhat.shape[0]
    Y = WOhat @ C
    gj = np.einsum("jt,jt->j", C, C)
    n2 = np.einsum("ij,ij->j", WOhat, WOhat)
    score = (n2 * gj).reshape(-1, g).sum(axis=1)
    mask, idx, tau = select_topk(score, k_heads, group=g)
    lam = delta * np.sum(gj) / C.shape[0]
    WO = refit_fc2(Y, C, idx, lam, d, C.shape[0])
    return dict(score=score, mask=mask, idx=idx, tau=tau, lam=lam, WO=WO, Y=Y)


# --------------------------------------------------------------------------------------
# Driver: Alg. 1 (temperature grid -> allocation -> per-module ADMM -> total loss)
# --------------------------------------------------------------------------------------
def prune_model(modules, rbar, temperatures, K, alpha=1.0, beta=1.0, delta=0.01,
                mode=WANDA, reselect=False):
    """modules: list of (W1hat, W2hat, X).  Returns per-temperature results and the best T."""
    results = {}
    for temp in temperatures:
        states = [module_init(W1, W2, X, delta) for (W1, W2, X) in modules]
        energies = [layer_energy(module_scores(st, mode)) for st in states]
        n_units = [st.W1hat.shape[0] for st in states]
        r, nprune = softmax_allocation(energies, n_units, rbar, temp)
        losses = []
        for st, npr, n in zip(states, nprune, n_units):
            k = int(n - npr)
            for it in range(K):
                terms = admm_step(st, k, alpha, beta, mode, select=(reselect or it == 0))
            losses.append(float(np.sum(terms)))
        results[temp] = dict(r=r, nprune=nprune, losses=losses, total=float(np.sum(losses)),
                             states=states, energies=energies)
    best = min(results, key=lambda t: results[t]["total"])
    return results, best


# --------------------------------------------------------------------------------------
# Brute force over channel subsets of the separable per-layer objective (eq. (78))
# --------------------------------------------------------------------------------------
def separable_objective(M, X, Z, Z0, A, A0, W2hat, second_term_only=False):
    """Phi(M) = sum_j |B_j - M_j C_j|^2 + |Y_j - M_j D_j|^2 evaluated from its definition.

    B_j = row j of Z X^+ X (b = W a with W = z a^+), C_j = Z0_j, D_j = W2hat[:,j] A_j (d x T),
    Y_j = W2hat[:,j] A0_j.
    """
    Pi = np.linalg.pinv(X) @ X
    B = Z @ Pi
    tot = 0.0
    for j in range(Z.shape[0]):
        if not second_term_only:
            tot += np.sum((B[j] - M[j] * Z0[j]) ** 2)
        Dj = np.outer(W2hat[:, j], A[j])
        Yj = np.outer(W2hat[:, j], A0[j])
        tot += np.sum((Yj - M[j] * Dj) ** 2)
    return tot


def brute_force_mask(k, X, Z, Z0, A, A0, W2hat, second_term_only=False):
    """Enumerate every subset of k kept units; return the best mask and its objective."""
    n = Z.shape[0]
    best, best_M = None, None
    for keep in itertools.combinations(range(n), k):
        M = np.zeros(n)
        M[list(keep)] = 1.0
        val = separable_objective(M, X, Z, Z0, A, A0, W2hat, second_term_only)
        if best is None or val < best:
            best, best_M = val, M
    return best_M.astype(np.uint8), best
