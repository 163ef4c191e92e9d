"""ctypes binding of libnadmm (include/nadmm.h).  Argument marshalling only.

PyTorch is used for device memory and streams; every step of the computation
runs in the library's HIP kernels.  There is no CPU fallback: if the shared
library has not been built (python -m paper_1807_07132_amd.build) loading fails
with an error.
"""
from __future__ import annotations

import ctypes as C
import math
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("NADMM_LIB", os.path.join(_HERE, "libnadmm.so"))  # NADMM_LIB: alternative build of the same library

NADMM_OK, NADMM_EINVAL, NADMM_EWORKSPACE, NADMM_EUNSUPPORTED, NADMM_EHIP, NADMM_ESCRATCH = 0, -1, -2, -3, -4, -5
NADMM_TRACE_LEN = 64
NADMM_MAX_LS = 62
NADMM_MAX_FREE_CLASSES = 32


class nadmm_sparse(C.Structure):
    _fields_ = [
        ("nnz", C.c_int64), ("d_row_ptr", C.c_void_p), ("d_col_idx", C.c_void_p), ("d_val", C.c_void_p),
        ("d_col_ptr", C.c_void_p), ("d_row_idx", C.c_void_p), ("d_val_t", C.c_void_p),
    ]


class nadmm_problem(C.Structure):
    _fields_ = [
        ("d_A", C.c_void_p), ("n", C.c_int64), ("p", C.c_int32), ("lda", C.c_int64),
        ("d_labels", C.c_void_p), ("C", C.c_int32), ("loss_scale", C.c_float),
        ("lambda_", C.c_float), ("rho", C.c_float), ("d_z", C.c_void_p), ("d_y", C.c_void_p),
        ("sparse", C.POINTER(nadmm_sparse)),
    ]


class SparseA:
    """Device-resident sparse storage of A: the row view (row_ptr int64 n+1, col_idx int32, val float32)
    and the column view (col_ptr int64 p+1, row_idx int32, val_t float32) of the same n x p matrix."""

    def __init__(self, n, p, row_ptr, col_idx, val, col_ptr, row_idx, val_t):
        self.shape = (int(n), int(p))
        self.nnz = int(val.numel())
        for t, dt, cnt in ((row_ptr, torch.int64, n + 1), (col_idx, torch.int32, self.nnz), (val, torch.float32, self.nnz),
                           (col_ptr, torch.int64, p + 1), (row_idx, torch.int32, self.nnz),
                           (val_t, torch.float32, self.nnz)):
            assert t.is_cuda and t.dtype == dt and t.is_contiguous() and t.numel() == cnt
        self.tensors = (row_ptr, col_idx, val, col_ptr, row_idx, val_t)
        self.device = val.device
        self.c = nadmm_sparse(self.nnz, *[t.data_ptr() for t in self.tensors])

    @classmethod
    def from_scipy(cls, csr, csc, device="cuda"):
        """Uploads a scipy.sparse CSR matrix and the CSC form of the same matrix (format conversion of the
        index types only)."""
        import numpy as np
        dev = torch.device(device)
        up = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a, dtype=dt)).to(dev)
        n, p = csr.shape
        assert csc.shape == csr.shape and csc.nnz == csr.nnz
        return cls(n, p, up(csr.indptr, np.int64), up(csr.indices, np.int32), up(csr.data, np.float32),
                   up(csc.indptr, np.int64), up(csc.indices, np.int32), up(csc.data, np.float32))


class nadmm_params(C.Structure):
    _fields_ = [
        ("max_newton", C.c_int32), ("max_cg", C.c_int32), ("max_ls", C.c_int32),
        ("cg_tol", C.c_float), ("grad_tol", C.c_float), ("armijo_beta", C.c_float),
        ("backtrack_gamma", C.c_float),
    ]


class nadmm_stats(C.Structure):
    _fields_ = [
        ("newton_iters", C.c_int32), ("cg_iters_total", C.c_int32), ("ls_evals_total", C.c_int32),
        ("armijo_failed", C.c_int32), ("loss_initial", C.c_double), ("loss_final", C.c_double),
        ("grad_norm_final", C.c_double), ("alpha", C.c_float * NADMM_TRACE_LEN),
        ("cg_iters", C.c_int32 * NADMM_TRACE_LEN), ("loss", C.c_double * NADMM_TRACE_LEN),
        ("grad_norm", C.c_double * NADMM_TRACE_LEN),
    ]


NADMM_MAX_WORKERS = 64


class nadmm_admm_params(C.Structure):
    _fields_ = [("max_outer", C.c_int32), ("eps_abs", C.c_float), ("eps_rel", C.c_float), ("local", nadmm_params),
                ("penalty_rule", C.c_int32), ("rb_mu", C.c_float), ("rb_tau", C.c_float)]


class nadmm_admm_stats(C.Structure):
    _fields_ = [
        ("outer_iters", C.c_int32), ("converged", C.c_int32), ("r_norm", C.c_double), ("d_norm", C.c_double),
        ("eps_pri", C.c_double), ("eps_dual", C.c_double), ("r_trace", C.c_double * NADMM_TRACE_LEN),
        ("d_trace", C.c_double * NADMM_TRACE_LEN), ("rho_scale", C.c_double),
        ("rho_scale_trace", C.c_double * NADMM_TRACE_LEN),
    ]


_lib = None


def lib():
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1807_07132_amd.build`; "
                           "there is no fallback path")
    L = C.CDLL(LIB_PATH)
    PP, PR, PS = C.POINTER(nadmm_problem), C.POINTER(nadmm_params), C.POINTER(nadmm_stats)
    vp, sz = C.c_void_p, C.c_size_t
    L.nadmm_version.restype = C.c_int
    L.nadmm_status_string.restype = C.c_char_p
    L.nadmm_status_string.argtypes = [C.c_int]
    L.nadmm_last_hip_error.restype = C.c_char_p
    L.nadmm_workspace_bytes.restype = sz
    L.nadmm_workspace_bytes.argtypes = [PP, PR]
    L.nadmm_loss_grad.argtypes = [PP, vp, vp, vp, vp, sz, vp]
    L.nadmm_hessvec.argtypes = [PP, vp, vp, vp, vp, sz, vp]
    L.nadmm_static_scratch_bytes.restype = sz
    L.nadmm_static_scratch_bytes.argtypes = []
    L.nadmm_hessvec_static_bytes.restype = sz
    L.nadmm_hessvec_static_bytes.argtypes = [PP]
    L.nadmm_hessvec_static.argtypes = [PP, vp, vp, vp, vp]
    L.nadmm_cg_solve.argtypes = [PP, vp, vp, vp, C.c_int, C.c_float, vp, vp, vp, sz, vp]
    L.nadmm_line_search.argtypes = [PP, vp, vp, vp, C.c_double, C.c_float, C.c_float, C.c_int, vp, vp, vp, vp, sz, vp]
    L.nadmm_local_newton.argtypes = [PP, vp, PR, PS, vp, sz, vp]
    PA, PAS = C.POINTER(nadmm_admm_params), C.POINTER(nadmm_admm_stats)
    L.nadmm_admm_workspace_bytes.restype = sz
    L.nadmm_admm_workspace_bytes.argtypes = [PP, C.c_int32, PA]
    L.nadmm_admm_consensus.argtypes = [C.c_int32, C.c_int64, vp, vp, vp, C.POINTER(C.c_float), C.c_float, C.c_float,
                                       C.c_float, vp, vp, sz, vp]
    L.nadmm_admm_solve.argtypes = [PP, C.c_int32, C.c_float, vp, vp, vp, PA, PAS, vp, sz, vp]
    L.nadmm_set_kernel_path.argtypes = [C.c_int]
    L.nadmm_query_kernel_path.argtypes = [PP]
    for f in (L.nadmm_loss_grad, L.nadmm_hessvec, L.nadmm_hessvec_static, L.nadmm_cg_solve, L.nadmm_line_search, L.nadmm_local_newton,
              L.nadmm_set_kernel_path, L.nadmm_query_kernel_path, L.nadmm_admm_consensus, L.nadmm_admm_solve):
        f.restype = C.c_int
    _lib = L
    return L


class NadmmError(RuntimeError):
    def __init__(self, code):
        self.code = code
        msg = lib().nadmm_status_string(code).decode()
        if code == NADMM_EHIP:
            msg += ": " + lib().nadmm_last_hip_error().decode()
        super().__init__(f"nadmm status {code}: {msg}")


def _check(code):
    if code != NADMM_OK:
        raise NadmmError(code)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


class Problem:
    """Device-resident data share.  Keeps the tensors alive and builds the C view."""

    def __init__(self, A, labels: Optional[torch.Tensor], C_: int, loss_scale: float, lam: float,
                 rho: float, z: Optional[torch.Tensor] = None, y: Optional[torch.Tensor] = None):
        """A: n x p float32 device tensor (rows contiguous), or a SparseA."""
        self.is_sparse = isinstance(A, SparseA)
        if not self.is_sparse:
            assert A.is_cuda and A.dtype == torch.float32 and A.dim() == 2 and A.stride(1) == 1
        self.A, self.labels, self.C, self.z, self.y = A, labels, int(C_), z, y
        self.n, self.p = A.shape
        self.NC = self.C - 1
        self.loss_scale, self.lam, self.rho = float(loss_scale), float(lam), float(rho)
        if labels is not None:
            assert labels.is_cuda and labels.dtype == torch.int32 and labels.numel() == self.n
        for t in (z, y):
            if t is not None:
                assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == self.p * self.NC
        self.c = nadmm_problem(None if self.is_sparse else A.data_ptr(), self.n, self.p,
                               self.p if self.is_sparse else A.stride(0),
                               labels.data_ptr() if labels is not None else None, self.C,
                               self.loss_scale, self.lam, self.rho,
                               z.data_ptr() if z is not None else None, y.data_ptr() if y is not None else None,
                               C.pointer(A.c) if self.is_sparse else None)
        self._ws = None

    @classmethod
    def from_workload(cls, w, device="cuda"):
        dev = torch.device(device)
        to = lambda a: torch.from_numpy(a).to(dev)
        A = SparseA.from_scipy(w.A, w.extra["csc"], dev) if w.sparse else to(w.A)
        return cls(A, to(w.b), w.C, w.s, w.lam, w.rho, to(w.z), to(w.y))

    def workspace(self, params=None) -> torch.Tensor:
        """Cached workspace for this problem, sized for `params` (nadmm_workspace_bytes) and regrown if a later call needs more."""
        need = nadmm_workspace_bytes(self, params)
        if need == 0:
            raise NadmmError(NADMM_EINVAL)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.A.device)
        return self._ws

    def vec(self) -> torch.Tensor:
        return torch.empty((self.p, self.NC), dtype=torch.float32, device=self.A.device)


def make_params(max_newton=10, max_cg=10, max_ls=10, cg_tol=0.0, grad_tol=0.0, armijo_beta=1e-4,
                backtrack_gamma=0.5) -> nadmm_params:
    return nadmm_params(max_newton, max_cg, max_ls, cg_tol, grad_tol, armijo_beta, backtrack_gamma)


def nadmm_version() -> int:
    return lib().nadmm_version()


def nadmm_workspace_bytes(prob: Problem, params: Optional[nadmm_params] = None) -> int:
    return int(lib().nadmm_workspace_bytes(C.byref(prob.c), C.byref(params) if params is not None else None))


def nadmm_set_kernel_path(path: int) -> int:
    rc = lib().nadmm_set_kernel_path(int(path))
    if rc < 0:
        raise NadmmError(rc)
    return rc


def nadmm_query_kernel_path(prob: Problem) -> int:
    rc = lib().nadmm_query_kernel_path(C.byref(prob.c))
    if rc < 0:
        raise NadmmError(rc)
    return rc


def nadmm_loss_grad(prob: Problem, X: torch.Tensor, want_grad=True, loss_out=None, grad_out=None, ws=None,
                    stream=None):
    """Returns (loss, grad): loss a float64 device scalar tensor, grad p x (C-1) float32 or None."""
    ws = prob.workspace() if ws is None else ws
    loss = torch.empty((), dtype=torch.float64, device=X.device) if loss_out is None else loss_out
    grad = (prob.vec() if grad_out is None else grad_out) if want_grad else None
    _check(lib().nadmm_loss_grad(C.byref(prob.c), _ptr(X), _ptr(loss), _ptr(grad), _ptr(ws), ws.numel(),
                                 _stream(stream)))
    return loss, grad


def nadmm_hessvec(prob: Problem, X: torch.Tensor, V: torch.Tensor, out=None, ws=None, stream=None):
    ws = prob.workspace() if ws is None else ws
    out = prob.vec() if out is None else out
    _check(lib().nadmm_hessvec(C.byref(prob.c), _ptr(X), _ptr(V), _ptr(out), _ptr(ws), ws.numel(), _stream(stream)))
    return out


def nadmm_hessvec_static(prob: Problem, X: torch.Tensor, V: torch.Tensor, out: torch.Tensor, stream=None):
    """nadmm_hessvec on the library's built-in scratch buffer; `out` is the caller's (nothing is allocated here)."""
    _check(lib().nadmm_hessvec_static(C.byref(prob.c), _ptr(X), _ptr(V), _ptr(out), _stream(stream)))
    return out


def nadmm_static_scratch_bytes() -> int:
    return int(lib().nadmm_static_scratch_bytes())


def nadmm_hessvec_static_bytes(prob: Problem) -> int:
    return int(lib().nadmm_hessvec_static_bytes(C.byref(prob.c)))


def nadmm_cg_solve(prob: Problem, X: torch.Tensor, g: torch.Tensor, max_iter: int, tol: float, out=None, ws=None,
                   stream=None):
    """Returns (p, iters, relres) as device tensors."""
    ws = prob.workspace() if ws is None else ws
    out = prob.vec() if out is None else out
    iters = torch.empty((), dtype=torch.int32, device=X.device)
    relres = torch.empty((), dtype=torch.float32, device=X.device)
    _check(lib().nadmm_cg_solve(C.byref(prob.c), _ptr(X), _ptr(g), _ptr(out), int(max_iter), float(tol),
                                _ptr(iters), _ptr(relres), _ptr(ws), ws.numel(), _stream(stream)))
    return out, iters, relres


def nadmm_line_search(prob: Problem, X: torch.Tensor, p: torch.Tensor, g: torch.Tensor, loss_at_X=math.nan,
                      beta=1e-4, gamma=0.5, max_ls=10, ws=None, stream=None):
    """Returns (alpha, loss_new, armijo_ok) as device scalar tensors."""
    ws = prob.workspace() if ws is None else ws
    alpha = torch.empty((), dtype=torch.float32, device=X.device)
    loss_new = torch.empty((), dtype=torch.float64, device=X.device)
    ok = torch.empty((), dtype=torch.int32, device=X.device)
    _check(lib().nadmm_line_search(C.byref(prob.c), _ptr(X), _ptr(p), _ptr(g), float(loss_at_X), float(beta),
                                   float(gamma), int(max_ls), _ptr(alpha), _ptr(loss_new), _ptr(ok), _ptr(ws),
                                   ws.numel(), _stream(stream)))
    return alpha, loss_new, ok


def nadmm_local_newton(prob: Problem, X: torch.Tensor, params: nadmm_params, want_stats=True, ws=None, stream=None):
    """Updates X in place.  Returns a dict of statistics (synchronises) or None."""
    ws = prob.workspace(params) if ws is None else ws
    st = nadmm_stats() if want_stats else None
    _check(lib().nadmm_local_newton(C.byref(prob.c), _ptr(X), C.byref(params), C.byref(st) if st is not None else None,
                                    _ptr(ws), ws.numel(), _stream(stream)))
    if st is None:
        return None
    k = min(st.newton_iters, NADMM_TRACE_LEN)
    return dict(newton_iters=st.newton_iters, cg_iters_total=st.cg_iters_total, ls_evals_total=st.ls_evals_total,
                armijo_failed=st.armijo_failed, loss_initial=st.loss_initial, loss_final=st.loss_final,
                grad_norm_final=st.grad_norm_final, alpha=list(st.alpha[:k]), cg_iters=list(st.cg_iters[:k]),
                loss=list(st.loss[:k]), grad_norm=list(st.grad_norm[:k]))


def make_admm_params(max_outer: int, local: nadmm_params, eps_abs=0.0, eps_rel=0.0, penalty_rule=0, rb_mu=10.0,
                     rb_tau=2.0) -> nadmm_admm_params:
    """penalty_rule 0: fixed penalties; 1: residual balancing with imbalance threshold rb_mu and factor rb_tau."""
    return nadmm_admm_params(int(max_outer), float(eps_abs), float(eps_rel), local, int(penalty_rule), float(rb_mu),
                             float(rb_tau))


def _worker_array(workers):
    arr = (nadmm_problem * len(workers))()
    for i, w in enumerate(workers):
        arr[i] = w.c
    return arr


def nadmm_admm_workspace_bytes(workers, params: Optional[nadmm_admm_params] = None) -> int:
    arr = _worker_array(workers)
    return int(lib().nadmm_admm_workspace_bytes(arr, len(workers), C.byref(params) if params is not None else None))


def nadmm_admm_consensus(x: torch.Tensor, u: torch.Tensor, z: torch.Tensor, rhos, lam: float, eps_abs=0.0, eps_rel=0.0,
                         ws=None, stream=None):
    """One z-/multiplier update on x (N x d), u (N x d, updated in place), z (d, updated in place).
    Returns a device tensor of 4 float64: ||r||, ||d||, eps_pri, eps_dual."""
    N, d = x.shape[0], x[0].numel()
    assert x.is_contiguous() and u.is_contiguous() and z.is_contiguous() and u.shape == x.shape and z.numel() == d
    out = torch.empty(4, dtype=torch.float64, device=x.device)
    ws = torch.empty(1 << 16, dtype=torch.uint8, device=x.device) if ws is None else ws
    rho_arr = (C.c_float * N)(*[float(r) for r in rhos])
    _check(lib().nadmm_admm_consensus(N, d, _ptr(x), _ptr(u), _ptr(z), rho_arr, float(lam), float(eps_abs),
                                      float(eps_rel), _ptr(out), _ptr(ws), ws.numel(), _stream(stream)))
    return out


def nadmm_admm_solve(workers, lam: float, x: torch.Tensor, params: nadmm_admm_params, want_stats=True, ws=None,
                     stream=None):
    """Algorithm 1 on the shards `workers` (Problem objects; rho of each is its penalty).  x: N x p x (C-1), warm
    starts in, local iterates out.  Returns (z, u, stats): u = multipliers in the sign convention of
    nadmm_problem.d_y (minus the paper's y)."""
    N = len(workers)
    assert x.is_contiguous() and x.shape[0] == N
    arr = _worker_array(workers)
    if ws is None:
        nbytes = int(lib().nadmm_admm_workspace_bytes(arr, N, C.byref(params)))
        if nbytes == 0:
            raise NadmmError(NADMM_EINVAL)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=x.device)
    u = torch.empty_like(x)
    z = torch.empty_like(x[0])
    st = nadmm_admm_stats() if want_stats else None
    _check(lib().nadmm_admm_solve(arr, N, float(lam), _ptr(x), _ptr(u), _ptr(z), C.byref(params),
                                  C.byref(st) if st is not None else None, _ptr(ws), ws.numel(), _stream(stream)))
    if st is None:
        return z, u, None
    k = min(st.outer_iters, NADMM_TRACE_LEN)
    return z, u, dict(outer_iters=st.outer_iters, converged=bool(st.converged), r_norm=st.r_norm, d_norm=st.d_norm,
                      eps_pri=st.eps_pri, eps_dual=st.eps_dual, r_trace=list(st.r_trace[:k]), d_trace=list(st.d_trace[:k]),
                      rho_scale=st.rho_scale, rho_scale_trace=list(st.rho_scale_trace[:k]))
