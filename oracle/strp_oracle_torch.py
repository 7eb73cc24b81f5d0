"""The FFN iteration of the numpy oracle once more in plain fp64 torch, token-chunked, for modules too large for numpy.

TEST INFRASTRUCTURE ONLY -- never imported by the product path, shares nothing with the HIP library.  Same definitions,
same order (Alg. 3 FFN function: score -> top-k -> refit fc2 -> refit fc1 -> a-update -> z-update -> objective), WANDA
score only.  Two things differ from strp_oracle.py, both forced by the size (an OPT-6.7B-shaped module has f x T = 4e9
auxiliaries):
  * every sum over the tokens is accumulated chunk by chunk (fp64 throughout), and Z0 / A0 are not kept;
  * the a-update solves the k x k system of the kept units, (alpha W_S^T W_S + beta I) A_S = alpha W_S^T Y + beta relu(Z_S),
    and sets A_j = relu(Z_j) on the pruned rows: the f x f system of Appendix A.1 with the pruned columns of W2 zero
    decouples into exactly these two parts.
It runs on whatever device its tensors live on (on a GPU the products go through the vendor's fp64 BLAS, not through
this repository's kernels).  tests/test_oracle_torch_pin.py holds it to strp_oracle.admm_step on the CPU.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

from . import strp_oracle as orc


@dataclass
class TorchState:
    X: torch.Tensor          # [d, >= T] input of fc1, any float dtype (converted per chunk)
    W1hat: torch.Tensor      # [f, d] fp64
    W2hat: torch.Tensor      # [d, f] fp64
    T: int
    Y: torch.Tensor          # [d, T] fp64
    H: torch.Tensor          # [d, d] fp64
    lam1: float
    lam2: float
    Z: torch.Tensor          # [f, T] fp64
    A: torch.Tensor          # [f, T] fp64
    W1: torch.Tensor = None  # [f, d] fp64, zero outside the kept rows
    W2: torch.Tensor = None  # [d, f] fp64, zero outside the kept columns
    mask: np.ndarray = None
    idx: torch.Tensor = None
    score: np.ndarray = None
    tau: float = float("nan")
    history: list = field(default_factory=list)


def _chunks(T, chunk):
    for t0 in range(0, T, chunk):
        yield t0, min(T, t0 + chunk)


def module_init(W1hat, W2hat, X, T, delta=0.01, chunk=8192) -> TorchState:
    """Alg. 3 initialisation: Z = Z0 = W1hat X, A = A0 = relu(Z0), Y = W2hat A0, H = X X^T, the two ridge weights."""
    dev = X.device
    W1 = W1hat.to(torch.float64)
    W2 = W2hat.to(torch.float64)
    f, d = W1.shape
    Z = torch.empty((f, T), dtype=torch.float64, device=dev)
    A = torch.empty((f, T), dtype=torch.float64, device=dev)
    Y = torch.empty((d, T), dtype=torch.float64, device=dev)
    H = torch.zeros((d, d), dtype=torch.float64, device=dev)
    a0sq = 0.0
    for t0, t1 in _chunks(T, chunk):
        Xc = X[:, t0:t1].to(torch.float64)
        Z[:, t0:t1] = W1 @ Xc
        A[:, t0:t1] = torch.relu(Z[:, t0:t1])
        Y[:, t0:t1] = W2 @ A[:, t0:t1]
        H += Xc @ Xc.T
        a0sq += float((A[:, t0:t1] ** 2).sum().item())
    lam1 = delta * float(torch.trace(H).item()) / d
    lam2 = delta * a0sq / f
    return TorchState(X=X, W1hat=W1, W2hat=W2, T=T, Y=Y, H=H, lam1=lam1, lam2=lam2, Z=Z, A=A)


def wanda_scores(st: TorchState, chunk=8192) -> np.ndarray:
    """n2_j sum_t A_jt^2 (square of eq. (wanda))."""
    g = torch.zeros(st.A.shape[0], dtype=torch.float64, device=st.A.device)
    for t0, t1 in _chunks(st.T, chunk):
        g += (st.A[:, t0:t1] ** 2).sum(dim=1)
    n2 = (st.W2hat ** 2).sum(dim=0)
    return (n2 * g).cpu().numpy()


def admm_step(st: TorchState, k, alpha=1.0, beta=1.0, select=True, chunk=8192):
    """One iteration; returns the five objective terms of strp_oracle.objective_terms."""
    dev = st.A.device
    f, d = st.W1hat.shape
    T = st.T
    if select or st.idx is None:
        score = wanda_scores(st, chunk)
        st.mask, idx, st.tau = orc.select_topk(score, k)       # the numpy oracle's selection rule itself
        st.score = score
        st.idx = torch.from_numpy(idx).to(dev)
    idx = st.idx
    kk = idx.numel()
    # ---- fc2: W2[:, S] = argmin |Y - W A_S|^2 + lam2 |W|^2
    G = torch.zeros((kk, kk), dtype=torch.float64, device=dev)
    R2 = torch.zeros((d, kk), dtype=torch.float64, device=dev)
    R1 = torch.zeros((kk, d), dtype=torch.float64, device=dev)
    for t0, t1 in _chunks(T, chunk):
        As = st.A[idx, t0:t1]
        G += As @ As.T
        R2 += st.Y[:, t0:t1] @ As.T
        R1 += st.Z[idx, t0:t1] @ st.X[:, t0:t1].to(torch.float64).T
    # the three systems are small (k x k, d x d): they are solved by numpy on the host, as in strp_oracle.py
    def host(t):
        return t.cpu().numpy()

    def back(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    W2s = back(np.linalg.solve(host(G) + st.lam2 * np.eye(kk), host(R2).T).T)
    st.W2 = torch.zeros((d, f), dtype=torch.float64, device=dev)
    st.W2[:, idx] = W2s
    # ---- fc1: W1[S, :] = argmin |Z_S - W X|^2 + lam1 |W|^2
    W1s = back(np.linalg.solve(host(st.H) + st.lam1 * np.eye(d), host(R1).T).T)
    st.W1 = torch.zeros((f, d), dtype=torch.float64, device=dev)
    st.W1[idx, :] = W1s
    # ---- a-update, then z-update, then the objective, chunk by chunk (each depends only on its own tokens).
    # The a-update's matrix alpha W_S^T W_S + beta I has its spectrum in [beta, beta + alpha |W_S|^2]: its inverse is
    # formed once and applied to every chunk's right-hand side.
    Minv = back(np.linalg.inv(alpha * (host(W2s).T @ host(W2s)) + beta * np.eye(kk)))
    pruned = torch.from_numpy(np.nonzero(st.mask == 0)[0]).to(dev)
    t1s = t2s = t3s = 0.0
    for t0, t1 in _chunks(T, chunk):
        Zc = st.Z[:, t0:t1]
        Yc = st.Y[:, t0:t1]
        Ac = torch.empty_like(Zc)
        rhs = alpha * (W2s.T @ Yc) + beta * torch.relu(Zc[idx])
        Ac[idx] = Minv @ rhs
        Ac[pruned] = torch.relu(Zc[pruned])
        Z1 = torch.zeros_like(Zc)
        Z1[idx] = W1s @ st.X[:, t0:t1].to(torch.float64)
        Z2 = (beta * Ac + alpha * Z1) / (alpha + beta)
        cm = torch.clamp(Z1, max=0.0)
        cost_m = beta * Ac * Ac + alpha * (cm - Z1) ** 2
        cp = torch.clamp(Z2, min=0.0)
        cost_p = beta * (Ac - cp) ** 2 + alpha * (cp - Z1) ** 2
        Zn = torch.where(cost_m < cost_p, cm, cp)
        t1s += float(((Yc - W2s @ Ac[idx]) ** 2).sum().item())
        t2s += float(((Ac - torch.relu(Zn)) ** 2).sum().item())
        t3s += float(((Zn - Z1) ** 2).sum().item())
        st.A[:, t0:t1] = Ac
        st.Z[:, t0:t1] = Zn
        del Ac, Z1, Z2, cm, cp, cost_m, cost_p, Zn, rhs
    terms = np.array([alpha * t1s, beta * t2s, alpha * t3s, alpha * st.lam2 * float((W2s ** 2).sum().item()),
                      alpha * st.lam1 * float((W1s ** 2).sum().item())]) / T
    st.history.append(terms)
    return terms
