"""The token-chunked torch form of the oracle's FFN iteration against the numpy oracle itself (CPU, fp64)."""
import numpy as np
import pytest
import torch

from oracle import strp_oracle as orc
from oracle import strp_oracle_torch as ort
from paper_2510_03246_amd import inputs


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


@pytest.mark.parametrize("reselect", [False, True])
@pytest.mark.parametrize("d,f,T,k,chunk", [(24, 96, 777, 40, 100), (40, 72, 256, 71, 256), (16, 64, 130, 1, 64)])
def test_chunked_torch_oracle_equals_the_numpy_oracle(d, f, T, k, chunk, reselect):
    """Three iterations side by side (ragged last chunk, one chunk, k = f - 1, k = 1): every sum over the tokens is only
    re-associated and the a-update only restricted to the kept block, so the two agree to rounding."""
    base = inputs.CONFIGS["tiny"]
    cfg = type(base)(**{**base.__dict__, "d": d, "f": f, "T": T})
    m = inputs.make_ffn_module(cfg, 0, 5, "cpu")
    W1, W2, X = (m[n].double() for n in ("W1hat", "W2hat", "X"))
    st_np = orc.module_init(W1.numpy(), W2.numpy(), X[:, :T].numpy())
    st_t = ort.module_init(m["W1hat"], m["W2hat"], m["X"], T, chunk=chunk)
    assert np.isclose(st_t.lam1, st_np.lam1, rtol=1e-13) and np.isclose(st_t.lam2, st_np.lam2, rtol=1e-13)
    assert rel(st_t.Y.numpy(), st_np.Y) < 1e-14 and rel(st_t.H.numpy(), st_np.H) < 1e-14
    for it in range(3):
        sel = reselect or it == 0
        t_np = orc.admm_step(st_np, k, 1.0, 0.7, orc.WANDA, select=sel)
        t_t = ort.admm_step(st_t, k, 1.0, 0.7, select=sel, chunk=chunk)
        assert np.array_equal(st_t.mask, st_np.mask)
        assert np.allclose(t_t, t_np, rtol=1e-9, atol=1e-14), (it, t_t, t_np)
        for name in ("W1", "W2", "Z", "A"):
            assert rel(getattr(st_t, name).numpy(), getattr(st_np, name)) < 1e-9, (it, name)
