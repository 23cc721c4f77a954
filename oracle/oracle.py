"""ctypes front-end of the C oracle (oracle/cals_oracle.c).  TEST INFRASTRUCTURE.

All arrays are numpy float64.  Tensors are C-contiguous of shape (I_N, ..., I2, I1) (first index
fastest in memory), N = 3 ... MAX_MODES; factor matrices are (I_n, R), converted to column-major on
the way in and returned Fortran-ordered.  Order-3 tensors go to the C routines without a suffix,
higher orders to the ones ending in _nd.  Nothing here imports or calls the GPU package.
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build

RUNNING, CONVERGED, MAX_ITERS, NUMERICAL = 0, 1, 2, 3
FLAG_NONNEG, FLAG_LINESEARCH = 1, 2
MAX_RANK = 32
MAX_MODES = 6
RANK_TOL = 1e-12

__all__ = ["RUNNING", "CONVERGED", "MAX_ITERS", "NUMERICAL", "FLAG_NONNEG", "FLAG_LINESEARCH", "MAX_RANK", "MAX_MODES", "RANK_TOL",
           "num_threads", "norm_sq", "gram", "hadamard", "cholesky", "cholesky_definite", "pinv_sym", "cholesky_solve", "mttkrp", "mttkrp_element",
           "nnls_row", "Model", "cp_als", "cals"]

_lib = None
_dp = C.POINTER(C.c_double)
_i64p = C.POINTER(C.c_int64)
_i32p = C.POINTER(C.c_int32)
_u32p = C.POINTER(C.c_uint32)


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        L.oracle_num_threads.restype = C.c_int
        L.oracle_norm_sq.restype = C.c_double
        L.oracle_norm_sq.argtypes = [_dp, _i64p]
        L.oracle_gram.argtypes = [_dp, C.c_int64, C.c_int, _dp]
        L.oracle_hadamard.argtypes = [_dp, _dp, C.c_int, _dp]
        L.oracle_cholesky.restype = C.c_int
        L.oracle_cholesky.argtypes = [_dp, C.c_int, _dp]
        L.oracle_cholesky_solve.argtypes = [_dp, C.c_int, _dp]
        L.oracle_mttkrp.argtypes = [_dp, _i64p, C.c_int, C.c_int64, _dp, _dp, _dp, _dp]
        L.oracle_mttkrp_element.argtypes = [_dp, _i64p, C.c_int, _dp, _dp, _dp, C.c_int64, C.c_int64, _dp, _dp]
        L.oracle_nnls_row.restype = C.c_int
        L.oracle_nnls_row.argtypes = [_dp, _dp, C.c_int, _dp, _u32p]
        L.oracle_model_create.restype = C.c_void_p
        L.oracle_model_create.argtypes = [_i64p, C.c_int, _dp, _dp, _dp, C.c_double, C.c_int, C.c_uint32, C.c_double]
        L.oracle_model_destroy.argtypes = [C.c_void_p]
        L.oracle_model_iterate.restype = C.c_int
        L.oracle_model_iterate.argtypes = [C.c_void_p, _dp, C.c_double]
        L.oracle_model_get.argtypes = [C.c_void_p, _dp, _dp, _dp, _dp, _dp, _dp, _i32p, _i32p, _i32p]
        L.oracle_model_last_ls_errors.restype = None
        L.oracle_model_last_ls_errors.argtypes = [C.c_void_p, _dp, _dp]
        L.oracle_cals.restype = C.c_int64
        L.oracle_cals.argtypes = [_dp, _i64p, C.c_int, _i32p, C.POINTER(_dp), _dp, _i32p, _u32p, _dp, C.c_int64,
                                  C.c_int, C.POINTER(_dp), _dp, _dp, _dp, _i32p, _i32p, _i32p, _i32p, C.c_int64]
        L.oracle_cholesky_definite.restype = C.c_int
        L.oracle_cholesky_definite.argtypes = [_dp, C.c_int, _dp]
        L.oracle_pinv_sym.restype = C.c_int
        L.oracle_pinv_sym.argtypes = [_dp, C.c_int, _dp, C.POINTER(C.c_int)]
        _pp = C.POINTER(_dp)
        L.oracle_norm_sq_nd.restype = C.c_double
        L.oracle_norm_sq_nd.argtypes = [_dp, C.c_int, _i64p]
        L.oracle_mttkrp_nd.argtypes = [_dp, C.c_int, _i64p, C.c_int, C.c_int64, _pp, _dp]
        L.oracle_mttkrp_element_nd.argtypes = [_dp, C.c_int, _i64p, C.c_int, _pp, C.c_int64, C.c_int64, _dp, _dp]
        L.oracle_model_create_nd.restype = C.c_void_p
        L.oracle_model_create_nd.argtypes = [C.c_int, _i64p, C.c_int, _pp, C.c_double, C.c_int, C.c_uint32, C.c_double]
        L.oracle_model_get_nd.argtypes = [C.c_void_p, _pp, _dp, _dp, _dp, _i32p, _i32p, _i32p]
        L.oracle_cals_nd.restype = C.c_int64
        L.oracle_cals_nd.argtypes = [_dp, C.c_int, _i64p, C.c_int, _i32p, _pp, _dp, _i32p, _u32p, _dp, C.c_int64,
                                     C.c_int, _pp, _dp, _dp, _dp, _i32p, _i32p, _i32p, _i32p, C.c_int64]
        _lib = L
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(_dp)


def _tensor(T: np.ndarray):
    assert T.dtype == np.float64 and 3 <= T.ndim <= MAX_MODES and T.flags.c_contiguous
    dims = np.array(T.shape[::-1], dtype=np.int64)
    return T, dims


def _ptrs(mats):
    return (_dp * len(mats))(*[_p(u) for u in mats])


def _f(U: np.ndarray) -> np.ndarray:
    return np.asfortranarray(U, dtype=np.float64)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def norm_sq(T: np.ndarray) -> float:
    T, dims = _tensor(T)
    if T.ndim != 3:
        return float(lib().oracle_norm_sq_nd(_p(T), T.ndim, dims.ctypes.data_as(_i64p)))
    return float(lib().oracle_norm_sq(_p(T), dims.ctypes.data_as(_i64p)))


def gram(U: np.ndarray) -> np.ndarray:
    U = _f(U)
    G = np.zeros((U.shape[1], U.shape[1]), order="F")
    lib().oracle_gram(_p(U), U.shape[0], U.shape[1], _p(G))
    return G


def hadamard(Ga: np.ndarray, Gb: np.ndarray) -> np.ndarray:
    Ga, Gb = _f(Ga), _f(Gb)
    H = np.zeros_like(Ga, order="F")
    lib().oracle_hadamard(_p(Ga), _p(Gb), Ga.shape[0], _p(H))
    return H


def cholesky(H: np.ndarray):
    H = _f(H)
    L = np.zeros_like(H, order="F")
    rc = lib().oracle_cholesky(_p(H), H.shape[0], _p(L))
    return rc, L


def cholesky_definite(H: np.ndarray):
    """Cholesky with the relative pivot test of the plain update: (1, .) when H is numerically rank-deficient."""
    H = _f(H)
    L = np.zeros_like(H, order="F")
    rc = lib().oracle_cholesky_definite(_p(H), H.shape[0], _p(L))
    return rc, L


def pinv_sym(H: np.ndarray):
    """(rc, P, rank): pseudo-inverse of a symmetric positive semi-definite matrix by Jacobi eigen-decomposition."""
    H = _f(H)
    P = np.zeros_like(H, order="F")
    k = C.c_int(0)
    rc = lib().oracle_pinv_sym(_p(H), H.shape[0], _p(P), C.byref(k))
    return rc, P, k.value


def cholesky_solve(L: np.ndarray, b: np.ndarray) -> np.ndarray:
    L = _f(L)
    x = np.array(b, dtype=np.float64).copy()
    lib().oracle_cholesky_solve(_p(L), L.shape[0], _p(x))
    return x


def mttkrp(T: np.ndarray, U: Sequence[np.ndarray], mode: int) -> np.ndarray:
    """Mode-`mode` (1..N) MTTKRP by definition; U are (I_n, R) with any common R (fused or not)."""
    T, dims = _tensor(T)
    Uf = [_f(u) for u in U]
    R = Uf[0].shape[1]
    assert len(Uf) == T.ndim and 1 <= mode <= T.ndim
    for n in range(T.ndim):
        assert Uf[n].shape == (dims[n], R)
    M = np.zeros((int(dims[mode - 1]), R), order="F")
    if T.ndim != 3:
        lib().oracle_mttkrp_nd(_p(T), T.ndim, dims.ctypes.data_as(_i64p), mode, R, _ptrs(Uf), _p(M))
        return M
    lib().oracle_mttkrp(_p(T), dims.ctypes.data_as(_i64p), mode, R, _p(Uf[0]), _p(Uf[1]), _p(Uf[2]), _p(M))
    return M


def mttkrp_element(T: np.ndarray, U: Sequence[np.ndarray], mode: int, row: int, col: int):
    """(value, sum of |terms|) of one MTTKRP element, accumulated in extended precision."""
    T, dims = _tensor(T)
    Uf = [_f(u) for u in U]
    v, a = C.c_double(), C.c_double()
    if T.ndim != 3:
        lib().oracle_mttkrp_element_nd(_p(T), T.ndim, dims.ctypes.data_as(_i64p), mode, _ptrs(Uf), int(row), int(col),
                                       C.byref(v), C.byref(a))
        return v.value, a.value
    lib().oracle_mttkrp_element(_p(T), dims.ctypes.data_as(_i64p), mode, _p(Uf[0]), _p(Uf[1]), _p(Uf[2]),
                                int(row), int(col), C.byref(v), C.byref(a))
    return v.value, a.value


def nnls_row(H: np.ndarray, m: np.ndarray, passive: int = 0):
    H = _f(H)
    m = np.ascontiguousarray(m, dtype=np.float64)
    x = np.zeros(H.shape[0])
    P = C.c_uint32(passive)
    rc = lib().oracle_nnls_row(_p(H), _p(m), H.shape[0], _p(x), C.byref(P))
    return rc, x, int(P.value)


class Model:
    """One CP-ALS instance that can be advanced an iteration at a time."""

    def __init__(self, T: np.ndarray, init: Sequence[np.ndarray], tol: float = -1.0, max_iters: int = 50,
                 flags: int = 0, alpha: float = 1.0, normT2: Optional[float] = None):
        self.T, self.dims = _tensor(T)
        self.R = int(init[0].shape[1])
        U = [_f(u) for u in init]
        self.normT2 = norm_sq(T) if normT2 is None else float(normT2)
        assert len(U) == self.T.ndim
        if self.T.ndim != 3:
            self.h = lib().oracle_model_create_nd(self.T.ndim, self.dims.ctypes.data_as(_i64p), self.R, _ptrs(U),
                                                  float(tol), int(max_iters), int(flags), float(alpha))
        else:
            self.h = lib().oracle_model_create(self.dims.ctypes.data_as(_i64p), self.R, _p(U[0]), _p(U[1]), _p(U[2]),
                                               float(tol), int(max_iters), int(flags), float(alpha))
        if not self.h:
            raise ValueError("rank out of range")

    def iterate(self) -> int:
        return int(lib().oracle_model_iterate(self.h, _p(self.T), self.normT2))

    def last_ls_errors(self):
        """(error after the iteration, error of the extrapolated point) as compared by the last line-search decision;
        NaNs before the first."""
        a, b = C.c_double(), C.c_double()
        lib().oracle_model_last_ls_errors(self.h, C.byref(a), C.byref(b))
        return a.value, b.value

    def state(self, factors: bool = True) -> dict:
        if not factors:
            fit, err = C.c_double(), C.c_double()
            it, st, acc = C.c_int32(), C.c_int32(), C.c_int32()
            if self.T.ndim != 3:
                lib().oracle_model_get_nd(self.h, None, None, C.byref(fit), C.byref(err), C.byref(it), C.byref(st), C.byref(acc))
            else:
                lib().oracle_model_get(self.h, None, None, None, None, C.byref(fit), C.byref(err), C.byref(it),
                                       C.byref(st), C.byref(acc))
            return dict(fit=fit.value, err=err.value, iters=it.value, status=st.value, ls_accepted=acc.value)
        U = [np.zeros((int(self.dims[n]), self.R), order="F") for n in range(self.T.ndim)]
        lam = np.zeros(self.R)
        fit, err = C.c_double(), C.c_double()
        it, st, acc = C.c_int32(), C.c_int32(), C.c_int32()
        if self.T.ndim != 3:
            lib().oracle_model_get_nd(self.h, _ptrs(U), _p(lam), C.byref(fit), C.byref(err), C.byref(it), C.byref(st),
                                      C.byref(acc))
        else:
            lib().oracle_model_get(self.h, _p(U[0]), _p(U[1]), _p(U[2]), _p(lam), C.byref(fit), C.byref(err),
                                   C.byref(it), C.byref(st), C.byref(acc))
        return dict(U=U, lam=lam, fit=fit.value, err=err.value, iters=it.value, status=st.value,
                    ls_accepted=acc.value)

    def __del__(self):
        if getattr(self, "h", None):
            lib().oracle_model_destroy(self.h)
            self.h = None


def cp_als(T: np.ndarray, init: Sequence[np.ndarray], tol: float = -1.0, max_iters: int = 50, flags: int = 0,
           alpha: float = 1.0) -> dict:
    """Plain CP-ALS for one starting point; returns final state plus the fit after every iteration."""
    m = Model(T, init, tol, max_iters, flags, alpha)
    hist = []
    while True:
        st = m.iterate()
        s = m.state()
        if st != NUMERICAL:
            hist.append(s["fit"])
        if st != RUNNING:
            break
    s["fit_history"] = np.array(hist)
    return s


def cals(T: np.ndarray, models: Sequence[dict], max_total_rank: int, max_slots: int = 0, max_rounds: int = 1 << 16) -> dict:
    """Full CALS (queue in, lock-step iterations, queue out).  `models` are dicts with rank, init,
    tol, max_iters, flags, ls_alpha, in enqueue order."""
    T, dims = _tensor(T)
    n = len(models)
    ranks = np.array([m["rank"] for m in models], dtype=np.int32)
    tol = np.array([m["tol"] for m in models], dtype=np.float64)
    mit = np.array([m["max_iters"] for m in models], dtype=np.int32)
    flg = np.array([m.get("flags", 0) for m in models], dtype=np.uint32)
    alp = np.array([m.get("ls_alpha", 1.0) for m in models], dtype=np.float64)
    ins = [[_f(u) for u in m["init"]] for m in models]
    N = T.ndim
    outs = [[np.zeros((int(dims[k]), int(r)), order="F") for k in range(N)] for r in ranks]
    assert all(len(trip) == N for trip in ins)
    in_ptrs = (_dp * (N * n))(*[_p(u) for trip in ins for u in trip])
    out_ptrs = (_dp * (N * n))(*[_p(u) for trip in outs for u in trip])
    lam = np.zeros((n, MAX_RANK))
    fit = np.zeros(n)
    err = np.zeros(n)
    iters = np.zeros(n, dtype=np.int32)
    status = np.zeros(n, dtype=np.int32)
    order = np.full(n, -1, dtype=np.int32)
    rlog = np.zeros(max_rounds, dtype=np.int32)
    tail = (in_ptrs, _p(tol), mit.ctypes.data_as(_i32p), flg.ctypes.data_as(_u32p), _p(alp), int(max_total_rank),
            int(max_slots), out_ptrs, _p(lam), _p(fit), _p(err), iters.ctypes.data_as(_i32p),
            status.ctypes.data_as(_i32p), order.ctypes.data_as(_i32p), rlog.ctypes.data_as(_i32p), int(max_rounds))
    if N != 3:
        rounds = lib().oracle_cals_nd(_p(T), N, dims.ctypes.data_as(_i64p), n, ranks.ctypes.data_as(_i32p), *tail)
    else:
        rounds = lib().oracle_cals(_p(T), dims.ctypes.data_as(_i64p), n, ranks.ctypes.data_as(_i32p), *tail)
    if rounds < 0:
        raise ValueError("bad model list (rank out of range or larger than max_total_rank)")
    return dict(U=outs, lam=[lam[k, :ranks[k]].copy() for k in range(n)], fit=fit, err=err, iters=iters,
                status=status, retire_order=order, rounds=int(rounds), total_rank_log=rlog[:min(rounds, max_rounds)])
