"""ctypes binding of the C-ABI in include/cals.h: argument marshalling only.

PyTorch is used for device memory and streams (the tensor and the multi-matrices handed to
cals_mttkrp are torch CUDA tensors; the library enqueues on torch's current stream).  There is no
Python or CPU implementation of any step here: without the built HIP library every call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))

FLAG_NONNEG, FLAG_LINESEARCH = 1, 2
CTX_TIMING = 1
CTX_REUSE = 2
RUNNING, CONVERGED, MAX_ITERS, NUMERICAL = 0, 1, 2, 3
E_TOOLARGE = -7
NOALLOC_SCRATCH_BYTES = 256 << 20
MAX_RANK = 32
MAX_MODES = 6

EXPORTS = ["cals_create", "cals_destroy", "cals_submit_tensor", "cals_submit_tensor_nd", "cals_enqueue_model", "cals_iterate", "cals_run",
           "cals_poll_retired", "cals_get_factors", "cals_mttkrp", "cals_mttkrp_noalloc", "cals_mttkrp_reuse", "cals_mttkrp_reuse_nd", "cals_get_round_log", "cals_get_stats", "cals_yardstick",
           "cals_strerror"]


class CalsError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__("%s failed: %s (%d)" % (what, _strerror(code), code))
        self.code = code


class _Options(C.Structure):
    _fields_ = [("max_total_rank", C.c_int64), ("max_slots", C.c_int32), ("device", C.c_int32),
                ("stream", C.c_void_p), ("flags", C.c_uint32)]


class _Result(C.Structure):
    _fields_ = [("model_id", C.c_int64), ("rank", C.c_int32), ("iters", C.c_int32), ("status", C.c_int32),
                ("ls_accepted", C.c_int32), ("fit", C.c_double), ("error", C.c_double)]


class _RoundRecord(C.Structure):
    _fields_ = [("round", C.c_int64), ("n_active", C.c_int32), ("total_rank", C.c_int32), ("ms", C.c_double),
                ("mttkrp_flops", C.c_double)]


class _Stats(C.Structure):
    _fields_ = [("rounds", C.c_int64), ("models_retired", C.c_int64), ("models_queued", C.c_int64),
                ("n_active", C.c_int32), ("total_rank", C.c_int32), ("tensor_norm_sq", C.c_double),
                ("mttkrp_flops", C.c_double), ("mttkrp_ms", C.c_double * MAX_MODES), ("reduce_ms", C.c_double * MAX_MODES),
                ("mttkrp_launches", C.c_int64 * MAX_MODES), ("mttkrp_rows_launches", C.c_int64)]


@dataclass
class Result:
    model_id: int
    rank: int
    iters: int
    status: int
    ls_accepted: int
    fit: float
    error: float


@dataclass
class Stats:
    rounds: int
    models_retired: int
    models_queued: int
    n_active: int
    total_rank: int
    tensor_norm_sq: float
    mttkrp_flops: float
    mttkrp_ms: List[float]
    reduce_ms: List[float]
    mttkrp_launches: List[int]
    mttkrp_rows_launches: int = 0


_lib: Optional[C.CDLL] = None
_dp = C.POINTER(C.c_double)


def library_path() -> str:
    return os.path.join(HERE, "libcals_hip.so")


def load_library() -> C.CDLL:
    """Load the built HIP library.  Never builds, never falls back: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise ImportError("HIP library %s is not built; run `python -m paper_2010_04678_amd.build` "
                          "(there is no CPU fallback)" % path)
    L = C.CDLL(path)
    vp = C.c_void_p
    L.cals_create.argtypes = [C.POINTER(vp), C.POINTER(_Options)]
    L.cals_destroy.argtypes = [vp]
    L.cals_submit_tensor.argtypes = [vp, vp, C.POINTER(C.c_int64), C.c_int]
    L.cals_submit_tensor_nd.argtypes = [vp, vp, C.c_int32, C.POINTER(C.c_int64), C.c_int]
    L.cals_enqueue_model.argtypes = [vp, C.c_int32, C.POINTER(vp), C.c_double, C.c_int32, C.c_uint32, C.c_double,
                                     C.POINTER(C.c_int64)]
    L.cals_iterate.argtypes = [vp, C.c_int32, C.POINTER(C.c_int32)]
    L.cals_run.argtypes = [vp]
    L.cals_poll_retired.argtypes = [vp, C.POINTER(_Result), C.c_int32, C.POINTER(C.c_int32)]
    L.cals_get_factors.argtypes = [vp, C.c_int64, C.POINTER(vp), vp]
    L.cals_mttkrp.argtypes = [vp, C.c_int32, C.c_int32, C.c_int64, C.POINTER(vp), vp]
    L.cals_mttkrp_noalloc.argtypes = [vp, C.c_int32, C.c_int32, C.c_int64, C.POINTER(vp), vp]
    L.cals_mttkrp_reuse.argtypes = [vp, C.c_int32, C.c_int64, C.POINTER(vp), vp, vp]
    L.cals_mttkrp_reuse_nd.argtypes = [vp, C.c_int32, C.c_int64, C.POINTER(vp), C.POINTER(vp)]
    L.cals_get_round_log.argtypes = [vp, C.c_int64, C.POINTER(_RoundRecord), C.c_int32, C.POINTER(C.c_int32)]
    L.cals_get_stats.argtypes = [vp, C.POINTER(_Stats)]
    L.cals_yardstick.argtypes = [vp, C.c_int32, vp, C.c_int64, C.c_int32, C.POINTER(C.c_double)]
    L.cals_strerror.argtypes = [C.c_int]
    L.cals_strerror.restype = C.c_char_p
    for name in EXPORTS:
        if name != "cals_strerror":
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


def _strerror(code: int) -> str:
    try:
        return load_library().cals_strerror(code).decode()
    except Exception:
        return "error"


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise CalsError(rc, what)


class Context:
    """One tensor, one queue of models (cals_ctx).  Methods mirror the C calls one to one."""

    def __init__(self, max_total_rank: int, max_slots: int = 0, device: int = 0, stream: Optional[int] = None,
                 flags: int = 0):
        self._L = load_library()
        if stream is None:
            import torch
            stream = torch.cuda.current_stream(device).cuda_stream
        opt = _Options(int(max_total_rank), int(max_slots), int(device), C.c_void_p(int(stream)), int(flags))
        h = C.c_void_p()
        _check(self._L.cals_create(C.byref(h), C.byref(opt)), "cals_create")
        self._h = h
        self.dims = None
        self._keep = []          # borrowed device tensors must outlive the context
        self._ranks = {}

    def close(self) -> None:
        if getattr(self, "_h", None):
            self._L.cals_destroy(self._h)
            self._h = None
            self._keep = []

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- cals_submit_tensor
    def submit_tensor(self, T) -> None:
        """T: torch CUDA float64 tensor (borrowed) or numpy array (copied), shape (I_N, ..., I2, I1) C-contiguous,
        i.e. first index fastest: element (i1,i2,i3) of an order-3 tensor at i1 + I1*(i2 + I2*i3).  Order 3 goes
        through cals_submit_tensor, higher orders through cals_submit_tensor_nd."""
        shape = tuple(int(d) for d in T.shape)
        nd = len(shape)
        dims = (C.c_int64 * nd)(*shape[::-1])
        if isinstance(T, np.ndarray):
            assert T.dtype == np.float64 and T.flags.c_contiguous
            ptr, on_device = T.ctypes.data, 0
        else:
            import torch
            assert T.is_cuda and T.dtype == torch.float64 and T.is_contiguous()
            self._keep.append(T)
            ptr, on_device = T.data_ptr(), 1
        if nd == 3:
            _check(self._L.cals_submit_tensor(self._h, ptr, dims, on_device), "cals_submit_tensor")
        else:
            _check(self._L.cals_submit_tensor_nd(self._h, ptr, nd, dims, on_device), "cals_submit_tensor_nd")
        self.dims = shape[::-1]

    # -- cals_enqueue_model
    def enqueue_model(self, init: Sequence[np.ndarray], tol: float = -1.0, max_iters: int = 50, flags: int = 0,
                      ls_alpha: float = 1.0) -> int:
        U = [np.asfortranarray(u, dtype=np.float64) for u in init]
        rank = int(U[0].shape[1])
        if self.dims is not None:           # without a tensor the library answers CALS_E_STATE itself
            if len(U) != len(self.dims):
                raise ValueError("init has %d matrices, the tensor %d modes" % (len(U), len(self.dims)))
            for n in range(len(self.dims)):
                if U[n].shape != (self.dims[n], rank):
                    raise ValueError("init[%d] has shape %s, expected %s" % (n, U[n].shape, (self.dims[n], rank)))
        ptrs = (C.c_void_p * len(U))(*[u.ctypes.data for u in U])
        mid = C.c_int64(-1)
        _check(self._L.cals_enqueue_model(self._h, rank, ptrs, float(tol), int(max_iters), int(flags),
                                          float(ls_alpha), C.byref(mid)), "cals_enqueue_model")
        self._ranks[mid.value] = rank
        return mid.value

    # -- cals_iterate / cals_run
    def iterate(self, n_rounds: int = 1) -> int:
        n = C.c_int32(0)
        _check(self._L.cals_iterate(self._h, int(n_rounds), C.byref(n)), "cals_iterate")
        return n.value

    def run(self) -> None:
        _check(self._L.cals_run(self._h), "cals_run")

    # -- cals_poll_retired
    def poll_retired(self, cap: int = 1024) -> List[Result]:
        buf = (_Result * cap)()
        n = C.c_int32(0)
        _check(self._L.cals_poll_retired(self._h, buf, cap, C.byref(n)), "cals_poll_retired")
        return [Result(r.model_id, r.rank, r.iters, r.status, r.ls_accepted, r.fit, r.error) for r in buf[:n.value]]

    # -- cals_get_factors
    def get_factors(self, model_id: int):
        rank = self._ranks[model_id]
        U = [np.zeros((self.dims[n], rank), order="F") for n in range(len(self.dims))]
        lam = np.zeros(rank)
        ptrs = (C.c_void_p * len(U))(*[u.ctypes.data for u in U])
        _check(self._L.cals_get_factors(self._h, int(model_id), ptrs, lam.ctypes.data), "cals_get_factors")
        return U, lam

    # -- cals_mttkrp
    def mttkrp(self, mode: int, U_dev: Sequence, M_dev, total_rank: Optional[int] = None, no_alloc: bool = False) -> None:
        """U_dev[n]: torch CUDA float64 (I_n, ld) row-major multi-matrices (the one for `mode` may be None);
        M_dev: (I_mode, ld), columns [0,total_rank) overwritten.  no_alloc: through cals_mttkrp_noalloc (fixed
        scratch array, nothing allocated)."""
        ld = int(M_dev.shape[1])
        tr = int(total_rank) if total_rank is not None else ld
        ptrs = (C.c_void_p * len(self.dims))()
        for n in range(len(self.dims)):
            u = U_dev[n]
            if u is None:
                ptrs[n] = None
                continue
            assert u.is_cuda and u.is_contiguous() and u.shape[1] == ld and u.shape[0] == self.dims[n]
            ptrs[n] = u.data_ptr()
        assert M_dev.is_cuda and M_dev.is_contiguous() and M_dev.shape[0] == self.dims[mode - 1]
        if no_alloc:
            _check(self._L.cals_mttkrp_noalloc(self._h, int(mode), tr, ld, ptrs, M_dev.data_ptr()), "cals_mttkrp_noalloc")
            return
        _check(self._L.cals_mttkrp(self._h, int(mode), tr, ld, ptrs, M_dev.data_ptr()), "cals_mttkrp")

    # -- cals_mttkrp_reuse
    def mttkrp_reuse(self, U_dev: Sequence, M2_dev, M3_dev, total_rank: Optional[int] = None) -> None:
        """Mode-2 and mode-3 MTTKRPs through the contraction of the tensor with U_dev[0] (two-step sweep)."""
        ld = int(M2_dev.shape[1])
        tr = int(total_rank) if total_rank is not None else ld
        ptrs = (C.c_void_p * 3)()
        for n in range(3):
            u = U_dev[n]
            assert u.is_cuda and u.is_contiguous() and u.shape[1] == ld and u.shape[0] == self.dims[n]
            ptrs[n] = u.data_ptr()
        assert M2_dev.is_cuda and M2_dev.is_contiguous() and M2_dev.shape[0] == self.dims[1]
        assert M3_dev.is_cuda and M3_dev.is_contiguous() and M3_dev.shape == (self.dims[2], ld)
        _check(self._L.cals_mttkrp_reuse(self._h, tr, ld, ptrs, M2_dev.data_ptr(), M3_dev.data_ptr()), "cals_mttkrp_reuse")

    # -- cals_mttkrp_reuse_nd
    def mttkrp_reuse_nd(self, U_dev: Sequence, M_dev: Sequence, total_rank: Optional[int] = None) -> None:
        """MTTKRPs of modes 2..N through the contraction of the tensor with U_dev[0]; M_dev[n] (I_n x ld) for n >= 1,
        M_dev[0] may be None."""
        N = len(self.dims)
        ld = int(M_dev[1].shape[1])
        tr = int(total_rank) if total_rank is not None else ld
        up = (C.c_void_p * N)()
        mp = (C.c_void_p * N)()
        for n in range(N):
            u = U_dev[n]
            assert u.is_cuda and u.is_contiguous() and u.shape == (self.dims[n], ld)
            up[n] = u.data_ptr()
            if n >= 1:
                m = M_dev[n]
                assert m.is_cuda and m.is_contiguous() and m.shape == (self.dims[n], ld)
                mp[n] = m.data_ptr()
        _check(self._L.cals_mttkrp_reuse_nd(self._h, tr, ld, up, mp), "cals_mttkrp_reuse_nd")

    # -- cals_yardstick
    def yardstick(self, kind: int, buf=None, reps: int = 5) -> float:
        """kind 0: fp64 MFMA issue rate (TFLOP/s); kind 1: streaming read of the CUDA tensor `buf` (GB/s)."""
        v = C.c_double(0.0)
        ptr = C.c_void_p(buf.data_ptr()) if buf is not None else None
        nbytes = int(buf.numel() * buf.element_size()) if buf is not None else 0
        _check(self._L.cals_yardstick(self._h, int(kind), ptr, C.c_int64(nbytes), int(reps), C.byref(v)), "cals_yardstick")
        return v.value

    # -- cals_get_round_log
    def round_log(self, first_round: int = 0, cap: int = 1 << 16):
        """[(round, n_active, total_rank, ms, mttkrp_flops), ...] for rounds first_round, first_round + 1, ..."""
        buf = (_RoundRecord * cap)()
        n = C.c_int32(0)
        _check(self._L.cals_get_round_log(self._h, int(first_round), buf, cap, C.byref(n)), "cals_get_round_log")
        return [(r.round, r.n_active, r.total_rank, r.ms, r.mttkrp_flops) for r in buf[:n.value]]

    # -- cals_get_stats
    def stats(self) -> Stats:
        s = _Stats()
        _check(self._L.cals_get_stats(self._h, C.byref(s)), "cals_get_stats")
        return Stats(s.rounds, s.models_retired, s.models_queued, s.n_active, s.total_rank, s.tensor_norm_sq,
                     s.mttkrp_flops, list(s.mttkrp_ms), list(s.reduce_ms), list(s.mttkrp_launches), int(s.mttkrp_rows_launches))


# ---- convenience driver in the spirit of the paper's cp_cals interface (Sec. 5, "interfaces") -----------------
def suggest_max_total_rank(ranks: Sequence[int], plateau: int = 256) -> int:
    """R* for a queue of models (Sec. 4, choice of the buffer size): the fused MTTKRP reaches its efficiency plateau
    at a fused width of about `plateau` columns (measured: 128-256 on MI355X), and wider buffers only add memory and
    iterations spent on models that could have been retired; so R* is the plateau width, but never more than all
    models need together and never less than the widest model."""
    ranks = [int(r) for r in ranks]
    if not ranks or min(ranks) < 1:
        raise ValueError("ranks must be positive")
    return max(max(ranks), min(sum(ranks), int(plateau)))


def suggest_two_step(dims: Sequence[int], max_total_rank: int, budget_bytes: int = 64 << 30) -> bool:
    """Whether two-step sweeps (CTX_REUSE) pay off.  They replace N-2 of a sweep's N fused MTTKRPs by reads of an
    intermediate of I2*...*IN*ld doubles (about two passes over it per sweep) and add a few launches per round.
    Measured, order 3: 40 -> 28 ms per sweep on 1000^3 at width 420, 123 -> 222 models/s on the 4000x200x50 line-search
    queue job, 930 -> 1010 on 200^3, but 3440 -> 3270 on 32^3, where a round is launch-bound; order 4 (180^4)
    60 -> 41 ms per round, order 5 (60^5) 60 -> 50.  So: at least 2^20 tensor elements, an intermediate within
    `budget_bytes`, and two passes over it (at 4.5 TB/s) cheaper than the MTTKRPs they replace (each the larger of
    its flops at 60 TFLOP/s and one pass over the tensor at 5.5 TB/s) -- which fails when the first mode is short,
    e.g. 50x200x4000, whose intermediate is 13 times the tensor at width 640."""
    dims = [int(d) for d in dims]
    ld = (int(max_total_rank) + 15) // 16 * 16
    elems = 1
    for d in dims:
        elems *= d
    y_bytes = (elems // dims[0]) * ld * 8
    t_mttkrp = max(2.0 * ld * elems / 60e12, 8.0 * elems / 5.5e12)
    return (elems >= (1 << 20) and y_bytes <= int(budget_bytes)
            and 2.0 * y_bytes / 4.5e12 < (len(dims) - 2) * t_mttkrp)


def cp_cals(T, inits: Sequence[Sequence[np.ndarray]], tol: float = 1e-4, max_iters: int = 50, nonneg: bool = False,
            line_search: bool = False, ls_alpha: float = 1.2, max_total_rank: Optional[int] = None, max_slots: int = 0,
            two_step: Optional[bool] = None, reorder_modes: bool = False):
    """Runs one CP-ALS model per entry of `inits` (one factor matrix I_n x R_k per mode) concurrently on the tensor T
    (numpy (I_N, ..., I2, I1) C-contiguous, or a CUDA float64 torch tensor of that shape; N = 3 .. MAX_MODES) and
    returns, in the order of `inits`, a list of (Result, [U1, ..., UN], lambda).  Pure marshalling around the C calls.
    two_step: two-step sweeps (CTX_REUSE); None = decide by suggest_two_step.
    reorder_modes: hand the library a copy of the tensor with its modes sorted by decreasing length (ties keep their
    order) and return the factors in the caller's order.  A sweep then updates the longest mode first -- still CP-ALS,
    but a different sequence of updates than with the caller's order -- which is what the kernels like best: the
    long mode gives the first contraction its rows, and two-step sweeps need it in front (4000 x 200 x 50 runs 1.5
    times faster than 50 x 200 x 4000).  Costs one transposed copy of the tensor."""
    N = len(T.shape)
    dims = tuple(int(d) for d in T.shape)[::-1]
    order = list(range(N))
    if reorder_modes:
        order = sorted(range(N), key=lambda n: -dims[n])          # new mode j is the caller's mode order[j]
        if order != list(range(N)):
            axes = [N - 1 - order[j] for j in reversed(range(N))]  # storage axis of mode n is N-1-n
            if isinstance(T, np.ndarray):
                T = np.ascontiguousarray(np.transpose(T, axes))
            else:
                T = T.permute(*axes).contiguous()
            inits = [[u[order[j]] for j in range(N)] for u in inits]
            dims = tuple(dims[order[j]] for j in range(N))
    ranks = [int(u[0].shape[1]) for u in inits]
    rstar = int(max_total_rank) if max_total_rank is not None else suggest_max_total_rank(ranks)
    if two_step is None:
        two_step = suggest_two_step(dims, rstar)
    flags = (FLAG_NONNEG if nonneg else 0) | (FLAG_LINESEARCH if line_search else 0)
    ctx = Context(max_total_rank=rstar, max_slots=max_slots, flags=CTX_REUSE if two_step else 0)
    try:
        ctx.submit_tensor(T)
        ids = [ctx.enqueue_model(u, tol, max_iters, flags, ls_alpha) for u in inits]
        ctx.run()
        res = {r.model_id: r for r in ctx.poll_retired(len(ids) + 1)}
        out = []
        for k in ids:
            U, lam = ctx.get_factors(k)
            back = [None] * N
            for j in range(N):
                back[order[j]] = U[j]
            out.append((res[k], back, lam))
        return out
    finally:
        ctx.close()
