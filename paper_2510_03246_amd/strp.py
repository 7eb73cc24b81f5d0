"""ctypes binding of libstrp.so: same entry-point names, argument marshalling only.

Every computation happens in the HIP library.  PyTorch is used for device memory and the
stream handle.  If the library has not been built, loading fails with an error (there is no
fallback path).
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libstrp.so")

OK, EINVAL, ENOMEM, ENOTPD, ENONFINITE, EHIP, ESTATE = range(7)
BF16, F32 = 0, 1
WANDA, LEMMA, GAIN = 0, 1, 2
SIDE_FC1, SIDE_FC2 = 0, 1
PREC_FAST, PREC_SPLIT = 0, 1
PROD_GRAM, PROD_RHS2, PROD_RHS1, PROD_RESID, PROD_AUPD, PROD_ZUPD = range(6)
STAGE_SELECT, STAGE_REFIT2, STAGE_REFIT1, STAGE_AUPD, STAGE_ZUPD, STAGE_OBJ = 1, 2, 4, 8, 16, 32
STAGE_ALL = 63

EXPORTS = [
    "strp_create", "strp_destroy", "strp_last_error", "strp_set_precision", "strp_set_product_planes", "strp_set_workspace",
    "strp_poll", "strp_workspace_bytes", "strp_module_cache_bytes", "strp_profile_enable", "strp_profile_read", "strp_profile_launches", "strp_gram", "strp_score_alloc", "strp_mask_topk", "strp_mask_topk_static", "strp_topk_workspace_bytes", "strp_weight_energy", "strp_alloc_inverse", "strp_alloc_softmax",
    "strp_refit", "strp_module_init", "strp_admm_step",
]


class StrpError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"strp status {status}: {msg}")
        self.status = status


class ModuleDesc(C.Structure):
    _fields_ = [("d", C.c_int32), ("f", C.c_int32), ("T", C.c_int64), ("ldx", C.c_int64), ("lda", C.c_int64),
                ("x_dtype", C.c_int32), ("w_dtype", C.c_int32), ("k_max", C.c_int32)]


class ScoreIn(C.Structure):
    _fields_ = [("A", C.c_void_p), ("a_dtype", C.c_int32), ("Z", C.c_void_p), ("Z0", C.c_void_p), ("ld", C.c_int64),
                ("T", C.c_int64), ("n_channels", C.c_int32), ("group", C.c_int32), ("mode", C.c_int32),
                ("n2", C.c_void_p), ("What", C.c_void_p), ("w_dtype", C.c_int32), ("w_rows", C.c_int32),
                ("ldw", C.c_int64)]


class ModuleState(C.Structure):
    _fields_ = [("X", C.c_void_p), ("W1hat", C.c_void_p), ("W2hat", C.c_void_p), ("Z", C.c_void_p), ("A", C.c_void_p),
                ("Z0", C.c_void_p), ("Y", C.c_void_p), ("W1", C.c_void_p), ("W2", C.c_void_p), ("H", C.c_void_p),
                ("cholH", C.c_void_p), ("n2", C.c_void_p), ("score", C.c_void_p), ("mask", C.c_void_p),
                ("idx", C.c_void_p), ("scalars", C.c_void_p), ("cache", C.c_void_p), ("s", C.c_int32), ("iter", C.c_int32),
                ("sums_cached", C.c_int32), ("precision", C.c_int32)]


class Params(C.Structure):
    _fields_ = [("alpha", C.c_double), ("beta", C.c_double), ("delta", C.c_double), ("mode", C.c_int32),
                ("reselect", C.c_int32), ("k", C.c_int32), ("stages", C.c_int32)]


class Report(C.Structure):
    _fields_ = [("terms", C.c_double * 5), ("J", C.c_double), ("J_ridge", C.c_double), ("lam1", C.c_double),
                ("lam2", C.c_double), ("tau", C.c_float), ("s", C.c_int32), ("status", C.c_int32)]


class WeightRef(C.Structure):
    _fields_ = [("W", C.c_void_p), ("dtype", C.c_int32), ("rows", C.c_int32), ("cols", C.c_int32), ("ld", C.c_int64)]


class ProfileEntry(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int32), ("ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


_lib = None


def load_library():
    """dlopen libstrp.so (built in-tree by paper_2510_03246_amd/build.py); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2510_03246_amd.build` "
                                "(or __graft_entry__.build()); there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_double
    lib.strp_create.argtypes = [C.POINTER(vp), C.c_int, vp]
    lib.strp_destroy.argtypes = [vp]
    lib.strp_last_error.argtypes = [vp]
    lib.strp_last_error.restype = C.c_char_p
    lib.strp_set_precision.argtypes = [vp, C.c_int]
    lib.strp_set_product_planes.argtypes = [vp, C.c_int, i32, i32]
    lib.strp_set_workspace.argtypes = [vp, vp, C.c_size_t]
    lib.strp_poll.argtypes = [vp]
    lib.strp_profile_enable.argtypes = [vp, C.c_int]
    lib.strp_profile_read.argtypes = [vp, C.POINTER(ProfileEntry), i32, C.POINTER(i32)]
    lib.strp_profile_launches.argtypes = [vp, C.POINTER(ProfileEntry), i32, C.POINTER(i32)]
    lib.strp_workspace_bytes.argtypes = [C.POINTER(ModuleDesc)]
    lib.strp_workspace_bytes.restype = C.c_size_t
    lib.strp_module_cache_bytes.argtypes = [C.POINTER(ModuleDesc)]
    lib.strp_module_cache_bytes.restype = C.c_size_t
    lib.strp_topk_workspace_bytes.restype = C.c_size_t
    lib.strp_topk_workspace_bytes.argtypes = [C.c_int32]
    lib.strp_weight_energy.argtypes = [vp, C.POINTER(WeightRef), i32, C.c_double, C.c_double, C.c_double, vp]
    lib.strp_alloc_inverse.argtypes = [vp, vp, i32, vp, vp, C.c_double, C.c_double, C.c_double, vp, vp]
    lib.strp_alloc_softmax.argtypes = [vp, vp, i32, vp, vp, C.c_double, C.c_double, C.c_double, vp, vp]
    lib.strp_gram.argtypes = [vp, vp, C.c_int, i32, i64, i64, vp, i32, vp, i32, vp, C.c_int]
    lib.strp_score_alloc.argtypes = [vp, C.POINTER(ScoreIn), vp, vp, i32, i32, vp, vp, dbl, dbl, dbl, vp, vp]
    lib.strp_mask_topk.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
    lib.strp_mask_topk_static.argtypes = [vp, vp, i32, i32, vp, vp, vp]
    lib.strp_refit.argtypes = [vp, C.c_int, vp, i32, dbl, vp, C.c_int, vp, C.c_int, i64, vp, C.c_int, i64, i64, vp,
                               i32, vp, i32, i32]
    lib.strp_module_init.argtypes = [vp, C.POINTER(ModuleDesc), C.POINTER(ModuleState), C.POINTER(Params)]
    lib.strp_admm_step.argtypes = [vp, C.POINTER(ModuleDesc), C.POINTER(ModuleState), C.POINTER(Params),
                                   C.POINTER(Report)]
    for name in EXPORTS:
        if name not in ("strp_last_error", "strp_workspace_bytes", "strp_module_cache_bytes", "strp_topk_workspace_bytes"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported dtype {t.dtype}")


class Context:
    """Owns a strp_ctx bound to torch's current stream on `device`, plus the caller-side workspace."""

    def __init__(self, device=0, workspace_bytes: int | None = None):
        self.lib = load_library()
        self.device = torch.device("cuda", device)
        torch.cuda.set_device(self.device)
        self.stream = torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        st = self.lib.strp_create(C.byref(h), device, C.c_void_p(self.stream.cuda_stream))
        if st != OK:
            raise StrpError(st, "strp_create failed")
        self.h = h
        self.ws = None
        if workspace_bytes:
            self.set_workspace(workspace_bytes)

    def close(self):
        if self.h:
            self.lib.strp_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def check(self, st):
        if st != OK:
            raise StrpError(st, self.lib.strp_last_error(self.h).decode())

    # ---- plumbing ---------------------------------------------------------------------
    def set_workspace(self, nbytes: int):
        self.ws = torch.empty(int(nbytes), dtype=torch.uint8, device=self.device)
        self.check(self.lib.strp_set_workspace(self.h, _ptr(self.ws), int(nbytes)))

    def ensure_workspace(self, nbytes: int):
        if self.ws is None or self.ws.numel() < nbytes:
            self.set_workspace(nbytes)

    def set_precision(self, prec: int):
        self.check(self.lib.strp_set_precision(self.h, prec))

    def set_product_planes(self, product: int, planes_p: int, planes_q: int):
        self.check(self.lib.strp_set_product_planes(self.h, product, planes_p, planes_q))

    def poll(self) -> int:
        return self.lib.strp_poll(self.h)

    def profile_enable(self, on: bool):
        self.check(self.lib.strp_profile_enable(self.h, int(on)))

    def profile_read(self):
        """Per-kernel-class totals since profile_enable: {name: dict(launches, ms, flops, bytes)}."""
        buf = (ProfileEntry * 64)()
        n = C.c_int32(0)
        self.check(self.lib.strp_profile_read(self.h, buf, 64, C.byref(n)))
        return {buf[i].name.decode(): dict(launches=buf[i].launches, ms=buf[i].ms, flops=buf[i].flops,
                                           bytes=buf[i].bytes) for i in range(n.value)}

    def profile_launches(self, max_entries: int = 4096):
        """The records since profile_enable one by one, in enqueue order: [(name, ms, flops, bytes), ...]."""
        buf = (ProfileEntry * max_entries)()
        n = C.c_int32(0)
        self.check(self.lib.strp_profile_launches(self.h, buf, max_entries, C.byref(n)))
        return [(buf[i].name.decode(), buf[i].ms, buf[i].flops, buf[i].bytes) for i in range(n.value)]

    def workspace_bytes(self, desc: ModuleDesc) -> int:
        return int(self.lib.strp_workspace_bytes(C.byref(desc)))

    # ---- entry points -------------------------------------------------------------------
    def strp_gram(self, A, T, idx=None, G=None, diag=None, accumulate=False, s=None):
        Crows, ldA = A.shape[0], A.stride(0)
        s = (idx.numel() if idx is not None else Crows) if s is None else s
        if G is None:
            G = torch.empty((s, s), dtype=torch.float32, device=A.device)
        self.check(self.lib.strp_gram(self.h, _ptr(A), dtype_code(A), Crows, T, ldA, _ptr(idx), s, _ptr(G),
                                      G.stride(0), _ptr(diag), int(accumulate)))
        return G

    def strp_score_alloc(self, A, T, mode, unit_score, energies, layer_idx, L, group=1, Z=None, Z0=None, n2=None,
                         What=None, n_units=None, group_id=None, rbar=0.5, temperature=1.0, rmax=0.95, r_out=None,
                         nprune_out=None):
        si = ScoreIn()
        si.A, si.a_dtype = A.data_ptr(), dtype_code(A)
        si.Z = Z.data_ptr() if Z is not None else None
        si.Z0 = Z0.data_ptr() if Z0 is not None else None
        si.ld, si.T, si.n_channels, si.group, si.mode = A.stride(0), T, A.shape[0], group, mode
        si.n2 = n2.data_ptr() if n2 is not None else None
        if What is not None:
            si.What, si.w_dtype, si.w_rows, si.ldw = What.data_ptr(), dtype_code(What), What.shape[0], What.stride(0)
        self.check(self.lib.strp_score_alloc(self.h, C.byref(si), _ptr(unit_score), _ptr(energies), layer_idx, L,
                                             _ptr(n_units), _ptr(group_id), rbar, temperature, rmax, _ptr(r_out),
                                             _ptr(nprune_out)))

    def strp_mask_topk(self, score, k, group=1, n=None):
        n = score.numel() if n is None else n
        mask = torch.empty(n, dtype=torch.uint8, device=score.device)
        idx = torch.empty(max(k * group, 1), dtype=torch.int32, device=score.device)
        tau = torch.empty(1, dtype=torch.float32, device=score.device)
        need = int(self.lib.strp_topk_workspace_bytes(n))
        if need:
            self.ensure_workspace(need)
        self.check(self.lib.strp_mask_topk(self.h, _ptr(score), n, k, group, _ptr(mask), _ptr(idx), _ptr(tau)))
        return mask, idx[: k * group], tau

    def strp_mask_topk_static(self, score, k, mask, idx, tau, n=None):
        """The allocation-free variant: every buffer, outputs included, is the caller's; nothing is allocated here."""
        n = score.numel() if n is None else n
        self.check(self.lib.strp_mask_topk_static(self.h, _ptr(score), n, k, _ptr(mask), _ptr(idx), _ptr(tau)))

    def strp_weight_energy(self, mats, var_coef, l2_coef, scale, energy):
        """energy (device double, 1 element) += scale (|W|_1 + var_coef Var(W) + l2_coef |W|_2) over the 2-D tensors in mats."""
        self.ensure_workspace(1 << 16)
        refs = (WeightRef * len(mats))()
        for r, m in zip(refs, mats):
            r.W, r.dtype, r.rows, r.cols, r.ld = m.data_ptr(), dtype_code(m), m.shape[0], m.shape[1], m.stride(0)
        self.check(self.lib.strp_weight_energy(self.h, refs, len(mats), float(var_coef), float(l2_coef), float(scale), _ptr(energy)))

    def strp_alloc_inverse(self, energies, n_units, rbar, temperature, rmax=0.95, group_id=None):
        L = energies.numel()
        r = torch.empty(L, dtype=torch.float64, device=energies.device)
        npr = torch.empty(L, dtype=torch.int32, device=energies.device)
        self.check(self.lib.strp_alloc_inverse(self.h, _ptr(energies), L, _ptr(n_units), _ptr(group_id), float(rbar),
                                               float(temperature), float(rmax), _ptr(r), _ptr(npr)))
        return r, npr

    def strp_alloc_softmax(self, energies, n_units, rbar, temperature, rmax=0.95, group_id=None):
        L = energies.numel()
        r = torch.empty(L, dtype=torch.float64, device=energies.device)
        npr = torch.empty(L, dtype=torch.int32, device=energies.device)
        self.check(self.lib.strp_alloc_softmax(self.h, _ptr(energies), L, _ptr(n_units), _ptr(group_id), float(rbar),
                                               float(temperature), float(rmax), _ptr(r), _ptr(npr)))
        return r, npr

    def strp_refit(self, side, Gram, lam, Lhs, Rhs, T, idx, W, chol=None, chol_valid=False):
        out, inn = W.shape
        self.check(self.lib.strp_refit(self.h, side, _ptr(Gram), Gram.stride(0) if Gram is not None else 0, float(lam),
                                       _ptr(chol), int(chol_valid), _ptr(Lhs), dtype_code(Lhs), Lhs.stride(0),
                                       _ptr(Rhs), dtype_code(Rhs), Rhs.stride(0), T, _ptr(idx), idx.numel(), _ptr(W),
                                       out, inn))
        return W

    def strp_module_init(self, desc, state, params):
        self.check(self.lib.strp_module_init(self.h, C.byref(desc), C.byref(state), C.byref(params)))

    def strp_admm_step(self, desc, state, params, report=True):
        rep = Report() if report else None
        self.check(self.lib.strp_admm_step(self.h, C.byref(desc), C.byref(state), C.byref(params),
                                           C.byref(rep) if rep is not None else None))
        return rep


class FFNModule:
    """Device buffers of one resident FFN module plus the ctypes structs that describe them."""

    def __init__(self, ctx: Context, W1hat: torch.Tensor, W2hat: torch.Tensor, X: torch.Tensor, T: int,
                 k_max: int = 0):
        dev = ctx.device
        f, d = W1hat.shape
        self.ctx, self.d, self.f, self.T = ctx, d, f, T
        self.W1hat, self.W2hat, self.X = W1hat.contiguous(), W2hat.contiguous(), X
        lda = (T + 7) // 8 * 8
        self.lda = lda
        e = lambda *shape, dt=torch.float32: torch.empty(shape, dtype=dt, device=dev)
        self.Z, self.A, self.Z0 = e(f, lda), e(f, lda), e(f, lda)
        self.Y = e(d, lda)
        self.W1, self.W2 = e(f, d), e(d, f)
        self.H = e(d, d)
        self.cholH = e(d, d, dt=torch.float64)
        self.n2 = e(f, dt=torch.float64)
        self.score = e(f)
        self.mask = e(f, dt=torch.uint8)
        self.idx = e(f, dt=torch.int32)
        self.scalars = torch.zeros(32, dtype=torch.float64, device=dev)
        self.desc = ModuleDesc(d, f, T, X.stride(0), lda, dtype_code(X), dtype_code(W1hat), k_max)
        self.cache = torch.empty(int(ctx.lib.strp_module_cache_bytes(C.byref(self.desc))), dtype=torch.uint8, device=dev)
        st = ModuleState()
        for name in ("X", "W1hat", "W2hat", "Z", "A", "Z0", "Y", "W1", "W2", "H", "cholH", "n2", "score", "mask",
                     "idx", "scalars", "cache"):
            setattr(st, name, getattr(self, name).data_ptr())
        st.s, st.iter = 0, 0
        self.state = st
        ctx.ensure_workspace(ctx.workspace_bytes(self.desc))

    def rebind_inputs(self, W1hat: torch.Tensor, W2hat: torch.Tensor, X: torch.Tensor):
        """Point the state at another module's inputs of the same shapes (the state buffers are reused; call init next)."""
        assert W1hat.shape == self.W1hat.shape and W2hat.shape == self.W2hat.shape and X.shape == self.X.shape
        assert W1hat.dtype == self.W1hat.dtype and X.dtype == self.X.dtype and X.stride(0) == self.X.stride(0)
        self.W1hat, self.W2hat, self.X = W1hat, W2hat, X
        for name in ("X", "W1hat", "W2hat"):
            setattr(self.state, name, getattr(self, name).data_ptr())

    def init(self, params: Params):
        self.ctx.strp_module_init(self.desc, self.state, params)

    def step(self, params: Params, report=True):
        return self.ctx.strp_admm_step(self.desc, self.state, params, report)

    @property
    def s(self):
        return int(self.state.s)
