"""Seeded generators: tensors in first-index-fastest order, and column-major starting points.

Random numbers come from numpy's Philox counter-based generator, keyed by (seed, stream), so
that any slab of a large tensor can be produced on its own and in any order.

Memory convention: a tensor T of dims (I1, I2, I3) is returned as a C-contiguous numpy array
of shape (I3, I2, I1), i.e. element (i1, i2, i3) sits at flat offset i1 + I1*(i2 + I2*i3); tensors of
higher order likewise (shape = dims reversed, first index fastest).
Factor matrices are returned Fortran-ordered with shape (I_n, R) (column-major, ld = I_n).
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from typing import List, Sequence, Tuple

import numpy as np

from .configs import WorkloadConfig


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def uniform_factors(dims: Sequence[int], rank: int, seed: int) -> List[np.ndarray]:
    """One Uniform[0,1) matrix (I_n x rank) per mode, column-major."""
    out = []
    for n, I in enumerate(dims):
        g = _rng(seed, n)
        out.append(np.asfortranarray(g.random((int(I), int(rank)))))
    return out


def random_tensor(dims: Sequence[int], seed: int, signed: bool = False) -> np.ndarray:
    """A dense tensor of iid entries (Uniform[0,1), or standard normal when signed)."""
    shape = tuple(int(d) for d in dims)[::-1]
    g = _rng(seed, 7)
    return g.standard_normal(shape) if signed else g.random(shape)


def low_rank_tensor(dims: Sequence[int], rank: int, seed: int, noise: float = 0.0) -> np.ndarray:
    """Order-N tensor (N = len(dims)) = sum of `rank` outer products of Uniform[0,1) vectors, plus Gaussian
    noise of std noise * rms(noise-free tensor).  Built mode by mode from the last index down."""
    F = uniform_factors(dims, rank, seed)
    acc = np.ascontiguousarray(F[-1])                    # (I_N, R)
    for U in F[-2::-1]:                                  # prepend faster modes: (..., I_n, R)
        acc = acc[..., None, :] * U
    T = np.ascontiguousarray(acc.sum(axis=-1))
    if noise > 0.0:
        sigma = noise * math.sqrt(_low_rank_norm_sq(F) / float(T.size))
        T += sigma * _rng(seed, 99).standard_normal(T.shape)
    return T


def low_rank_tensor_device(dims: Sequence[int], rank: int, seed: int, noise: float = 0.0, device: str = "cuda:0"):
    """The same kind of tensor as low_rank_tensor, built on the GPU with torch (sizes that would take minutes on the
    host): Uniform[0,1) factors from a torch generator seeded with `seed`, plus Gaussian noise of std
    noise * rms(noise-free tensor), added slab by slab.  Returns (tensor of shape dims reversed, list of factors)."""
    import torch
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed))
    F = [torch.rand((int(d), int(rank)), dtype=torch.float64, device=dev, generator=g) for d in dims]
    K = F[-1]
    for U in F[-2:0:-1]:                                     # Khatri-Rao product of modes N..2, mode 2 fastest
        K = (K[:, None, :] * U[None, :, :]).reshape(-1, int(rank))
    T = (K @ F[0].T).reshape(tuple(int(d) for d in dims)[::-1])
    del K
    if noise > 0.0:
        sigma = noise * float(T.pow(2).mean().sqrt())
        step = max(1, T.shape[0] // 8)
        for i in range(0, T.shape[0], step):
            T[i:i + step].add_(sigma * torch.randn(T[i:i + step].shape, dtype=torch.float64, device=dev, generator=g))
    return T, F


def _collinear_factor(I: int, R: int, c: float, seed: int, stream: int) -> np.ndarray:
    """I x R matrix with unit columns whose pairwise cosine is exactly c (up to rounding): an orthonormal basis
    (Gram-Schmidt of a seeded Gaussian matrix, each projection applied twice) times the transposed Cholesky factor of
    c 11^T + (1 - c) I.  Every sum is an exactly rounded one (math.fsum) and every product is element-wise, so the
    result does not depend on the host's linear-algebra library, thread count or vector width: expected values
    stored for this tensor stay valid on any machine."""
    g = _rng(seed, stream)
    G = g.standard_normal((I, R))
    Q = np.empty((I, R))
    for j in range(R):
        v = G[:, j].copy()
        for _ in range(2):
            for i in range(j):
                v -= math.fsum(Q[:, i] * v) * Q[:, i]
        Q[:, j] = v / math.sqrt(math.fsum(v * v))
    L = np.zeros((R, R))                                   # lower Cholesky factor, column by column
    for j in range(R):
        d = 1.0 - math.fsum(L[j, k] * L[j, k] for k in range(j))
        L[j, j] = math.sqrt(d)
        for i in range(j + 1, R):
            L[i, j] = (c - math.fsum(L[i, k] * L[j, k] for k in range(j))) / L[j, j]
    out = np.zeros((I, R), order="F")
    for j in range(R):
        for k in range(j + 1):                             # column j = sum_k Q[:, k] L[j, k], k ascending
            out[:, j] += Q[:, k] * L[j, k]
    return out


def _eem_factors(dims: Sequence[int], R: int, seed: int) -> List[np.ndarray]:
    """samples x emission x excitation: lognormal concentrations, Gaussian-peak spectra."""
    I1, I2, I3 = (int(d) for d in dims)
    g = _rng(seed, 0)
    conc = np.exp(g.standard_normal((I1, R)))
    em_c = g.uniform(0.15, 0.85, R) * I2
    em_w = g.uniform(0.05, 0.15, R) * I2
    ex_c = g.uniform(0.15, 0.85, R) * I3
    ex_w = g.uniform(0.08, 0.20, R) * I3
    x2 = np.arange(I2)[:, None]
    x3 = np.arange(I3)[:, None]
    em = np.exp(-0.5 * ((x2 - em_c[None, :]) / em_w[None, :]) ** 2)
    ex = np.exp(-0.5 * ((x3 - ex_c[None, :]) / ex_w[None, :]) ** 2)
    return [np.asfortranarray(conc), np.asfortranarray(em), np.asfortranarray(ex)]


def true_factors(cfg: WorkloadConfig) -> List[np.ndarray]:
    if cfg.kind == "uniform":
        return uniform_factors(cfg.dims, cfg.true_rank, cfg.tensor_seed)
    if cfg.kind == "eem":
        return _eem_factors(cfg.dims, cfg.true_rank, cfg.tensor_seed)
    if cfg.kind == "collinear":
        return [_collinear_factor(int(I), cfg.true_rank, cfg.collinearity, cfg.tensor_seed, n)
                for n, I in enumerate(cfg.dims)]
    raise ValueError(cfg.kind)


def _low_rank_norm_sq(F: Sequence[np.ndarray]) -> float:
    """Squared norm of the tensor with factors F, from the factor Gramians; exactly rounded sums (math.fsum) of
    element-wise products, so the value is the same on every machine."""
    R = F[0].shape[1]
    G = np.ones((R, R))
    for U in F:
        for r in range(R):
            for q in range(r, R):
                g = math.fsum(U[:, r] * U[:, q])
                G[r, q] *= g
                if q != r:
                    G[q, r] *= g
    return math.fsum(G.reshape(-1))


def make_tensor(cfg: WorkloadConfig, dims: Sequence[int] | None = None, threads: int = 8,
                out: np.ndarray | None = None) -> np.ndarray:
    """Low-rank tensor plus Gaussian noise of std eta * rms(noise-free tensor), slab by slab.

    `dims` may shrink the configuration (same recipe, smaller tensor) for quick tests.
    Every slab is accumulated component by component with element-wise products and sums (no library matrix
    product, whose order of additions depends on the host), so the tensor is bit-identical on every machine and
    expected values stored for it stay valid.
    """
    if dims is not None and tuple(dims) != tuple(cfg.dims):
        cfg = WorkloadConfig(**{**cfg.__dict__, "dims": tuple(int(d) for d in dims)})
    I1, I2, I3 = cfg.dims
    A, B, C = true_factors(cfg)
    sigma = cfg.noise * math.sqrt(_low_rank_norm_sq([A, B, C]) / (float(I1) * I2 * I3))
    T = out if out is not None else np.empty((I3, I2, I1), dtype=np.float64)
    assert T.shape == (I3, I2, I1) and T.dtype == np.float64 and T.flags.c_contiguous
    At = np.ascontiguousarray(A.T)
    R = At.shape[0]

    def slab(i3: int) -> None:
        S = T[i3]
        Bc = B * C[i3][None, :]
        np.multiply(Bc[:, 0:1], At[0:1, :], out=S)         # S[i2, i1] = sum_r B[i2,r] C[i3,r] A[i1,r], r ascending
        tmp = np.empty_like(S)
        for r in range(1, R):
            np.multiply(Bc[:, r:r + 1], At[r:r + 1, :], out=tmp)
            S += tmp
        if sigma > 0.0:
            S += sigma * _rng(cfg.noise_seed, i3 + 16).standard_normal((I2, I1))
        if cfg.clip_at_zero:
            np.maximum(S, 0.0, out=S)

    if I3 * I2 * I1 < (1 << 22) or threads <= 1:
        for i3 in range(I3):
            slab(i3)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(slab, range(I3)))
    return T


def make_inits(dims: Sequence[int], ranks: Sequence[int], seeds: Sequence[int]) -> List[List[np.ndarray]]:
    """Uniform[0,1) starting points, one (U1, U2, U3) triple per model."""
    return [uniform_factors(dims, r, s) for r, s in zip(ranks, seeds)]


def make_models(cfg: WorkloadConfig, dims: Sequence[int] | None = None) -> List[dict]:
    """Model descriptors in enqueue order: rank, init, tol, max_iters, flags, ls_alpha."""
    d = tuple(dims) if dims is not None else cfg.dims
    inits = make_inits(d, cfg.ranks, cfg.init_seeds)
    return [dict(model_id=m, rank=r, init=inits[m], tol=cfg.tol, max_iters=cfg.max_iters,
                 flags=cfg.flags, ls_alpha=cfg.ls_alpha) for m, r in enumerate(cfg.ranks)]
