"""ctypes binding over libbbmm.so -- argument marshalling only.

Every function mirrors one entry point of include/bbmm.h under the same name.  Device
arrays are torch CUDA (HIP) tensors; PyTorch is used only to own device memory and to
provide the stream.  There is no fallback: if the shared library is missing or a call
fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbbmm.so")

KERNEL_RBF, KERNEL_MATERN52 = 0, 1
MODE_MATERIALISED, MODE_ONTHEFLY, MODE_SGPR = 0, 1, 2
OK, EINVAL, ENOMEM, ENOTPD, ENONFINITE, EHIP, ENOCONV = 0, 1, 2, 3, 4, 5, 6
MAX_ITERS = 256

EXPORTS = [
    "bbmm_create", "bbmm_destroy", "bbmm_last_error", "bbmm_tune", "bbmm_mm_timing", "bbmm_loop_graph_stats",
    "bbmm_solve_logdet_grad",
    "bbmm_setup", "bbmm_build_khat", "bbmm_khat_block", "bbmm_sgpr_build", "bbmm_sgpr_root_rows",
    "bbmm_kernel_mm", "bbmm_pivoted_cholesky",
    "bbmm_precond_setup", "bbmm_precond_solve", "bbmm_make_probes", "bbmm_mbcg",
    "bbmm_tridiag_eig_batched", "bbmm_tridiag_eig_batched_noalloc", "bbmm_slq_logdet", "bbmm_slq_from_coeffs", "bbmm_dk_traces",
    "bbmm_predict_mean", "bbmm_predict_var",
]


class BbmmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("bbmm error %d: %s" % (code, msg))
        self.code = code


class _Problem(C.Structure):
    _fields_ = [("kernel", C.c_int32), ("mode", C.c_int32),
                ("n", C.c_int64), ("d", C.c_int64), ("t", C.c_int64), ("k", C.c_int64),
                ("max_iters", C.c_int64), ("tol", C.c_double),
                ("n_lengthscale", C.c_int64), ("lengthscale", C.POINTER(C.c_double)),
                ("outputscale", C.c_double), ("noise", C.c_double),
                ("X", C.c_void_p), ("y", C.c_void_p), ("E1", C.c_void_p), ("E2", C.c_void_p),
                ("m", C.c_int64), ("Uind", C.c_void_p), ("jitter_rel", C.c_double),
                ("pivots_in", C.POINTER(C.c_int64)), ("u0_init", C.c_void_p)]


class _Result(C.Structure):
    _fields_ = [("u0", C.c_void_p), ("U", C.c_void_p),
                ("logdet", C.c_double), ("logdet_precond", C.c_double), ("yKinvy", C.c_double),
                ("nlml", C.c_double),
                ("trace", C.POINTER(C.c_double)), ("quad", C.POINTER(C.c_double)),
                ("grad_nlml", C.POINTER(C.c_double)),
                ("iters_run", C.c_int64), ("rank", C.c_int64),
                ("alpha", C.POINTER(C.c_double)), ("beta", C.POINTER(C.c_double)),
                ("resid", C.POINTER(C.c_double)), ("pivots", C.POINTER(C.c_int64)),
                ("slq_terms", C.POINTER(C.c_double))]


_lib = None


def load_library() -> C.CDLL:
    """Loads libbbmm.so; raises if it has not been built (python -m paper_1809_11165_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError("%s not found: build it with `python -m paper_1809_11165_amd.build`"
                                % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    for name in EXPORTS:
        getattr(lib, name)            # AttributeError if a declared symbol is missing
    lib.bbmm_last_error.restype = C.c_char_p
    lib.bbmm_last_error.argtypes = [C.c_void_p]
    lib.bbmm_create.argtypes = [C.POINTER(C.c_void_p), C.c_int, C.c_void_p]
    lib.bbmm_destroy.argtypes = [C.c_void_p]
    lib.bbmm_tune.argtypes = [C.c_void_p, C.c_char_p, C.c_int64]
    lib.bbmm_mm_timing.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                   C.POINTER(C.c_int64)]
    lib.bbmm_loop_graph_stats.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    lib.bbmm_solve_logdet_grad.argtypes = [C.c_void_p, C.POINTER(_Problem), C.POINTER(_Result)]
    lib.bbmm_setup.argtypes = [C.c_void_p, C.POINTER(_Problem)]
    lib.bbmm_build_khat.argtypes = [C.c_void_p]
    lib.bbmm_khat_block.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_void_p]
    lib.bbmm_sgpr_build.argtypes = [C.c_void_p]
    lib.bbmm_sgpr_root_rows.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p]
    lib.bbmm_kernel_mm.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p]
    lib.bbmm_pivoted_cholesky.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int64),
                                          C.POINTER(C.c_int64)]
    lib.bbmm_precond_setup.argtypes = [C.c_void_p, C.POINTER(C.c_double)]
    lib.bbmm_precond_solve.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    lib.bbmm_make_probes.argtypes = [C.c_void_p, C.c_void_p]
    lib.bbmm_mbcg.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p,
                              C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double),
                              C.POINTER(C.c_int64)]
    lib.bbmm_tridiag_eig_batched.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                             C.c_int64, C.c_int64, C.POINTER(C.c_double),
                                             C.POINTER(C.c_double)]
    lib.bbmm_tridiag_eig_batched_noalloc.argtypes = lib.bbmm_tridiag_eig_batched.argtypes
    lib.bbmm_slq_logdet.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.bbmm_slq_from_coeffs.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                         C.POINTER(C.c_double), C.POINTER(C.c_int64), C.c_int64, C.c_int64,
                                         C.c_double, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.bbmm_dk_traces.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_double),
                                   C.POINTER(C.c_double)]
    lib.bbmm_predict_mean.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    lib.bbmm_predict_var.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p,
                                     C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    _lib = lib
    return lib


def _dptr(a):
    return C.c_void_p(a.ctypes.data) if isinstance(a, np.ndarray) else C.c_void_p(a.data_ptr())


def _dbl(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _check_dev(tensor, shape, name):
    import torch
    if not (isinstance(tensor, torch.Tensor) and tensor.is_cuda and tensor.dtype == torch.float32
            and tensor.is_contiguous()):
        raise TypeError("%s must be a contiguous float32 device tensor" % name)
    if tuple(tensor.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(tensor.shape), tuple(shape)))


@dataclass
class Problem:
    """Host description of one inference problem; X, y, E1, E2 are device tensors."""
    kernel: int
    mode: int
    X: "object"
    y: "object"
    lengthscale: np.ndarray
    outputscale: float
    noise: float
    E1: "object"
    E2: "object"
    k: int
    max_iters: int
    tol: float = 0.0
    Uind: "object" = None           # SGPR only: m x d device tensor of inducing inputs
    jitter_rel: float = 0.0         # SGPR only
    pivots_in: Optional[np.ndarray] = None   # replay this pivot order instead of the greedy rule
    u0_init: "object" = None                 # n device floats: warm start of the y column
    _keep: list = field(default_factory=list, repr=False)

    def to_c(self) -> _Problem:
        n, d = self.X.shape
        t = self.E2.shape[1]
        ls = np.ascontiguousarray(np.atleast_1d(self.lengthscale), dtype=np.float64)
        _check_dev(self.X, (n, d), "X")
        _check_dev(self.y, (n,), "y")
        _check_dev(self.E2, (n, t), "E2")
        if self.k > 0:
            _check_dev(self.E1, (self.k, t), "E1")
        self._keep = [ls]
        p = _Problem()
        p.kernel, p.mode = int(self.kernel), int(self.mode)
        p.n, p.d, p.t, p.k, p.max_iters = n, d, t, int(self.k), int(self.max_iters)
        p.tol = float(self.tol)
        p.n_lengthscale = ls.shape[0]
        p.lengthscale = _dbl(ls)
        p.outputscale, p.noise = float(self.outputscale), float(self.noise)
        p.X, p.y = self.X.data_ptr(), self.y.data_ptr()
        p.E1 = self.E1.data_ptr() if self.k > 0 else None
        p.E2 = self.E2.data_ptr()
        p.m, p.Uind, p.jitter_rel = 0, None, 0.0
        p.u0_init = None
        if self.u0_init is not None:
            _check_dev(self.u0_init, (n,), "u0_init")
            p.u0_init = self.u0_init.data_ptr()
        p.pivots_in = None
        if self.pivots_in is not None:
            piv = np.ascontiguousarray(self.pivots_in, dtype=np.int64)
            if piv.shape != (int(self.k),):
                raise ValueError("pivots_in must have k entries")
            self._keep.append(piv)
            p.pivots_in = piv.ctypes.data_as(C.POINTER(C.c_int64))
        if self.mode == MODE_SGPR:
            if self.Uind is None:
                raise ValueError("an SGPR problem needs Uind")
            _check_dev(self.Uind, (self.Uind.shape[0], d), "Uind")
            p.m, p.Uind, p.jitter_rel = int(self.Uind.shape[0]), self.Uind.data_ptr(), float(self.jitter_rel)
        return p


@dataclass
class Result:
    u0: "object"
    U: "object"
    logdet: float
    logdet_precond: float
    yKinvy: float
    nlml: float
    trace: np.ndarray
    quad: np.ndarray
    grad_nlml: np.ndarray
    iters_run: int
    rank: int
    alpha: np.ndarray
    beta: np.ndarray
    resid: np.ndarray
    pivots: np.ndarray
    slq_terms: np.ndarray
    estimator_rel_err: float = float("nan")   # filled by tests only


class Context:
    """Owns one bbmm_ctx bound to the current torch device and stream."""

    def __init__(self, device: int = 0, stream=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the BBMM path only runs on the HIP library")
        self.lib = load_library()
        self.torch = torch
        self.device = torch.device("cuda", device)
        self._stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        handle = C.c_void_p()
        rc = self.lib.bbmm_create(C.byref(handle), device, C.c_void_p(self._stream.cuda_stream))
        if rc != OK:
            raise BbmmError(rc, "bbmm_create failed")
        self.h = handle
        self._prob = None

    def close(self):
        if getattr(self, "h", None):
            self.lib.bbmm_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _ck(self, rc: int):
        if rc != OK:
            raise BbmmError(rc, self.lib.bbmm_last_error(self.h).decode())

    def _empty(self, *shape):
        return self.torch.empty(*shape, dtype=self.torch.float32, device=self.device)

    # ---- entry points (names follow include/bbmm.h) ------------------------------------
    def bbmm_tune(self, key: str, value: int):
        self._ck(self.lib.bbmm_tune(self.h, key.encode(), int(value)))

    def bbmm_mm_timing(self):
        """(average ms per K_hat.M launch, total ms, launches) of the last timed mBCG run."""
        avg, tot, cnt = C.c_double(0.0), C.c_double(0.0), C.c_int64(0)
        self._ck(self.lib.bbmm_mm_timing(self.h, C.byref(avg), C.byref(tot), C.byref(cnt)))
        return float(avg.value), float(tot.value), int(cnt.value)

    def bbmm_loop_graph_stats(self):
        """(graphs recorded, graphs replayed) by this context so far."""
        cap, rep = C.c_int64(0), C.c_int64(0)
        self._ck(self.lib.bbmm_loop_graph_stats(self.h, C.byref(cap), C.byref(rep)))
        return int(cap.value), int(rep.value)

    def bbmm_solve_logdet_grad(self, prob: Problem, want_U: bool = True) -> Result:
        p = prob.to_c()
        n, t, k, it = p.n, p.t, p.k, p.max_iters
        H = p.n_lengthscale + 2
        u0 = self._empty(n)
        U = self._empty(n, t + 1) if want_U else None
        trace, quad, grad = np.zeros(H), np.zeros(H), np.zeros(H)
        alpha, beta, resid = (np.zeros((it, t + 1)) for _ in range(3))
        pivots = np.full(max(k, 1), -1, dtype=np.int64)
        slq = np.zeros(t)
        r = _Result()
        r.u0 = u0.data_ptr()
        r.U = U.data_ptr() if want_U else None
        r.trace, r.quad, r.grad_nlml = _dbl(trace), _dbl(quad), _dbl(grad)
        r.alpha, r.beta, r.resid = _dbl(alpha), _dbl(beta), _dbl(resid)
        r.pivots = pivots.ctypes.data_as(C.POINTER(C.c_int64))
        r.slq_terms = _dbl(slq)
        self._ck(self.lib.bbmm_solve_logdet_grad(self.h, C.byref(p), C.byref(r)))
        self._prob = prob
        self._shape = (int(p.n), int(p.d), int(p.t), int(p.k), int(p.max_iters), int(p.n_lengthscale))
        return Result(u0=u0, U=U, logdet=r.logdet, logdet_precond=r.logdet_precond, yKinvy=r.yKinvy,
                      nlml=r.nlml, trace=trace, quad=quad, grad_nlml=grad, iters_run=int(r.iters_run),
                      rank=int(r.rank), alpha=alpha, beta=beta, resid=resid, pivots=pivots[:k],
                      slq_terms=slq)

    def bbmm_setup(self, prob: Problem):
        p = prob.to_c()
        self._ck(self.lib.bbmm_setup(self.h, C.byref(p)))
        self._prob = prob
        self._shape = (int(p.n), int(p.d), int(p.t), int(p.k), int(p.max_iters), int(p.n_lengthscale))

    def bbmm_build_khat(self):
        self._ck(self.lib.bbmm_build_khat(self.h))

    def bbmm_khat_block(self, row0: int, nrows: int, col0: int, ncols: int):
        out = self._empty(nrows, ncols)
        self._ck(self.lib.bbmm_khat_block(self.h, row0, nrows, col0, ncols, _dptr(out)))
        return out

    def bbmm_sgpr_build(self):
        self._ck(self.lib.bbmm_sgpr_build(self.h))

    def bbmm_sgpr_root_rows(self, row0: int, nrows: int):
        m = int(self._prob.Uind.shape[0])
        out = self._empty(nrows, m)
        self._ck(self.lib.bbmm_sgpr_root_rows(self.h, row0, nrows, _dptr(out)))
        return out

    def bbmm_kernel_mm(self, mode: int, M):
        n = self._shape[0]
        _check_dev(M, (n, M.shape[1]), "M")
        V = self._empty(n, M.shape[1])
        self._ck(self.lib.bbmm_kernel_mm(self.h, mode, _dptr(M), M.shape[1], _dptr(V)))
        return V

    def bbmm_pivoted_cholesky(self):
        n, _, _, k, _, _ = self._shape
        L = self.torch.empty(n, max(k, 1), dtype=self.torch.float64, device=self.device)
        piv = np.full(max(k, 1), -1, dtype=np.int64)
        rank = C.c_int64(0)
        self._ck(self.lib.bbmm_pivoted_cholesky(self.h, _dptr(L) if k > 0 else None,
                                                piv.ctypes.data_as(C.POINTER(C.c_int64)),
                                                C.byref(rank)))
        return L[:, :k], piv[:k], int(rank.value)

    def bbmm_precond_setup(self) -> float:
        out = C.c_double(0.0)
        self._ck(self.lib.bbmm_precond_setup(self.h, C.byref(out)))
        return float(out.value)

    def bbmm_precond_solve(self, R):
        n = self._shape[0]
        _check_dev(R, (n, R.shape[1]), "R")
        Z = self._empty(n, R.shape[1])
        self._ck(self.lib.bbmm_precond_solve(self.h, _dptr(R), R.shape[1], _dptr(Z)))
        return Z

    def bbmm_make_probes(self):
        n, _, t, _, _, _ = self._shape
        B = self._empty(n, t + 1)
        self._ck(self.lib.bbmm_make_probes(self.h, _dptr(B)))
        return B

    def bbmm_mbcg(self, mode: int, B):
        n, _, _, _, it, _ = self._shape
        c = B.shape[1]
        _check_dev(B, (n, c), "B")
        U = self._empty(n, c)
        alpha, beta, resid = (np.zeros((it, c)) for _ in range(3))
        iters = C.c_int64(0)
        self._ck(self.lib.bbmm_mbcg(self.h, mode, _dptr(B), c, _dptr(U), _dbl(alpha), _dbl(beta),
                                    _dbl(resid), C.byref(iters)))
        return U, alpha, beta, resid, int(iters.value)

    def bbmm_tridiag_eig_batched(self, diag: np.ndarray, off: np.ndarray, _fn=None):
        diag = np.ascontiguousarray(diag, dtype=np.float64)
        batch, m = diag.shape
        off = np.ascontiguousarray(off, dtype=np.float64).reshape(batch, max(m - 1, 0))
        vals, first = np.zeros((batch, m)), np.zeros((batch, m))
        offp = _dbl(off) if m > 1 else None
        fn = _fn if _fn is not None else self.lib.bbmm_tridiag_eig_batched
        self._ck(fn(self.h, _dbl(diag), offp, m, batch, _dbl(vals), _dbl(first)))
        return vals, first

    def bbmm_tridiag_eig_batched_noalloc(self, diag: np.ndarray, off: np.ndarray):
        return self.bbmm_tridiag_eig_batched(diag, off, _fn=self.lib.bbmm_tridiag_eig_batched_noalloc)

    def bbmm_slq_logdet(self):
        t = self._shape[2]
        out = C.c_double(0.0)
        terms = np.zeros(max(t, 1))
        self._ck(self.lib.bbmm_slq_logdet(self.h, C.byref(out), _dbl(terms)))
        return float(out.value), terms[:t]

    def bbmm_slq_from_coeffs(self, alpha: np.ndarray, beta: np.ndarray, rho0: np.ndarray, m_valid=None,
                             logdet_precond: float = 0.0):
        """alpha, beta: (p, t) coefficients of the probe columns; rho0: (t,); m_valid: (t,) or None."""
        alpha = np.ascontiguousarray(alpha, dtype=np.float64)
        beta = np.ascontiguousarray(beta, dtype=np.float64)
        rho0 = np.ascontiguousarray(rho0, dtype=np.float64)
        p, t = alpha.shape
        if beta.shape != (p, t) or rho0.shape != (t,):
            raise ValueError("alpha and beta must be (p, t), rho0 (t,)")
        mv = None
        mvp = None
        if m_valid is not None:
            mv = np.ascontiguousarray(m_valid, dtype=np.int64)
            if mv.shape != (t,):
                raise ValueError("m_valid must have t entries")
            mvp = mv.ctypes.data_as(C.POINTER(C.c_int64))
        out = C.c_double(0.0)
        terms = np.zeros(t)
        self._ck(self.lib.bbmm_slq_from_coeffs(self.h, _dbl(alpha), _dbl(beta), _dbl(rho0), mvp, p, t,
                                               float(logdet_precond), C.byref(out), _dbl(terms)))
        return float(out.value), terms

    def bbmm_dk_traces(self, U, W):
        n, _, t, _, _, nl = self._shape
        _check_dev(U, (n, t + 1), "U")
        _check_dev(W, (n, t), "W")
        trace, quad = np.zeros(nl + 2), np.zeros(nl + 2)
        self._ck(self.lib.bbmm_dk_traces(self.h, _dptr(U), _dptr(W), _dbl(trace), _dbl(quad)))
        return trace, quad

    def bbmm_predict_mean(self, Xstar, u0):
        n, d = self._shape[0], self._shape[1]
        ns = Xstar.shape[0]
        _check_dev(Xstar, (ns, d), "Xstar")
        _check_dev(u0, (n,), "u0")
        mean = self._empty(ns)
        self._ck(self.lib.bbmm_predict_mean(self.h, _dptr(Xstar), ns, _dptr(u0), _dptr(mean)))
        return mean

    def bbmm_predict_var(self, mode: int, Xstar):
        d = self._shape[1]
        ns = Xstar.shape[0]
        _check_dev(Xstar, (ns, d), "Xstar")
        var = self._empty(ns)
        iters, resid = C.c_int64(0), C.c_double(0.0)
        self._ck(self.lib.bbmm_predict_var(self.h, mode, _dptr(Xstar), ns, _dptr(var), C.byref(iters),
                                           C.byref(resid)))
        return var, int(iters.value), float(resid.value)


def problem_from_workload(w, mode: int, device="cuda:0") -> Problem:
    """Uploads a paper_1809_11165_amd.inputs.Workload (host arrays) and wraps it as a Problem."""
    import torch
    dev = torch.device(device)

    def up(a):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)

    E1 = up(w.E1) if w.k > 0 else None
    Uind = up(w.Uind) if mode == MODE_SGPR else None
    return Problem(kernel=w.kernel, mode=mode, X=up(w.X), y=up(w.y), lengthscale=w.lengthscale,
                   outputscale=w.outputscale, noise=w.noise, E1=E1, E2=up(w.E2), k=w.k,
                   max_iters=w.iters, tol=w.tol, Uind=Uind, jitter_rel=w.jitter_rel)
