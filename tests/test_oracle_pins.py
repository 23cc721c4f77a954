"""Pins for the CPU oracle: each test checks it against something other than itself -- brute
force, a closed form, an identity from the paper, or a library routine on a special case.

Citations name the paper's algorithms / equations / sections.
"""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.optimize

import oracle as O
from workloads import low_rank_tensor, random_tensor, uniform_factors

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def tview(T):
    """numpy view indexed [i1, i2, i3]."""
    return T.transpose(2, 1, 0)


def signed_factors(dims, R, seed):
    return [2.0 * u - 1.0 for u in uniform_factors(dims, R, seed)]


def reconstruct(U, lam=None):
    lam = np.ones(U[0].shape[1]) if lam is None else lam
    return np.einsum("r,ir,jr,kr->ijk", lam, U[0], U[1], U[2])


def krp(A, B):
    """Column-wise Kronecker product with A's row index the slow one (notation section)."""
    return np.einsum("ir,jr->ijr", A, B).reshape(A.shape[0] * B.shape[0], A.shape[1])


# ------------------------------------------------------------------ MTTKRP (Alg. 1, MTTKRP line)

@pytest.mark.parametrize("dims", [(5, 4, 3), (3, 5, 4), (1, 2, 3)])
def test_mttkrp_brute_force_triple_loop(dims):
    R = 2
    T = random_tensor(dims, 11, signed=True)
    U = signed_factors(dims, R, 12)
    Tn = tview(T)
    I1, I2, I3 = dims
    want = [np.zeros((I1, R)), np.zeros((I2, R)), np.zeros((I3, R))]
    for i1 in range(I1):
        for i2 in range(I2):
            for i3 in range(I3):
                for r in range(R):
                    t = Tn[i1, i2, i3]
                    want[0][i1, r] += t * U[1][i2, r] * U[2][i3, r]
                    want[1][i2, r] += t * U[0][i1, r] * U[2][i3, r]
                    want[2][i3, r] += t * U[0][i1, r] * U[1][i2, r]
    for mode in (1, 2, 3):
        got = O.mttkrp(T, U, mode)
        assert np.allclose(got, want[mode - 1], rtol=1e-13, atol=1e-14), mode


def test_mttkrp_is_unfolding_times_explicit_krp():
    # "the mode-n unfolding is multiplied with the Khatri-Rao product of all factor matrices except U(n)"
    dims, R = (17, 13, 11), 7
    T = random_tensor(dims, 21, signed=True)
    U = signed_factors(dims, R, 22)
    Tn = tview(T)
    T1 = Tn.reshape(dims[0], -1)                       # columns indexed (i2, i3), i2 slow
    T2 = Tn.transpose(1, 0, 2).reshape(dims[1], -1)    # (i1, i3)
    T3 = Tn.transpose(2, 0, 1).reshape(dims[2], -1)    # (i1, i2)
    want = [T1 @ krp(U[1], U[2]), T2 @ krp(U[0], U[2]), T3 @ krp(U[0], U[1])]
    for mode in (1, 2, 3):
        got = O.mttkrp(T, U, mode)
        scale = np.abs(want[mode - 1]).max()
        assert np.abs(got - want[mode - 1]).max() <= 1e-13 * scale * 50, mode


def test_mttkrp_of_modes_2_and_3_factor_through_the_mode_1_contraction():
    # the identity behind two-step sweeps (Sec. 2, partial-contraction reuse): with Y[i2,i3,c] = sum_i1 T U1,
    # M2[i2,c] = sum_i3 Y U3 and M3[i3,c] = sum_i2 Y U2 are the plain MTTKRPs of the oracle
    dims, R = (9, 7, 5), 4
    T = random_tensor(dims, 31, signed=True)
    U = signed_factors(dims, R, 32)
    Y = np.einsum("ijk,ic->jkc", tview(T), U[0])
    M2 = np.einsum("jkc,kc->jc", Y, U[2])
    M3 = np.einsum("jkc,jc->kc", Y, U[1])
    for mode, want in ((2, M2), (3, M3)):
        got = O.mttkrp(T, U, mode)
        assert np.abs(got - want).max() <= 1e-13 * np.abs(want).max() * 50, mode


def test_fused_mttkrp_column_blocks_equal_solo_results_bitwise():
    # Eq. (1)/(2): the fused MTTKRP of concatenated factors is the concatenation of the solo MTTKRPs.
    dims, ranks = (9, 8, 7), [1, 3, 2, 5, 11]
    T = random_tensor(dims, 31, signed=True)
    facs = [signed_factors(dims, r, 40 + k) for k, r in enumerate(ranks)]
    fused = [np.hstack([f[n] for f in facs]) for n in range(3)]
    for mode in (1, 2, 3):
        big = O.mttkrp(T, fused, mode)
        c = 0
        for f, r in zip(facs, ranks):
            solo = O.mttkrp(T, f, mode)
            assert np.array_equal(big[:, c:c + r], solo), (mode, r)
            c += r


def test_mttkrp_element_matches_exact_sum():
    dims, R = (6, 5, 4), 3
    T = random_tensor(dims, 51, signed=True)
    U = signed_factors(dims, R, 52)
    Tn = tview(T)
    for mode, row, col in [(1, 2, 1), (2, 4, 0), (3, 3, 2)]:
        terms = []
        for a in range(dims[0]):
            for b in range(dims[1]):
                for c in range(dims[2]):
                    idx = (a, b, c)
                    if idx[mode - 1] != row:
                        continue
                    others = [n for n in range(3) if n != mode - 1]
                    k = U[others[0]][idx[others[0]], col] * U[others[1]][idx[others[1]], col]
                    terms.append(Tn[a, b, c] * k)
        v, sa = O.mttkrp_element(T, U, mode, row, col)
        assert abs(v - math.fsum(terms)) <= 4e-16 * math.fsum(abs(t) for t in terms)
        assert abs(sa - math.fsum(abs(t) for t in terms)) <= 1e-15 * sa
        assert abs(O.mttkrp(T, U, mode)[row, col] - v) <= 1e-14 * sa


# ------------------------------------------------------------------ Gram / Hadamard / solve

def test_gram_of_khatri_rao_is_hadamard_of_grams():
    # Alg. 1, Hadamard line: (A kr B)^T (A kr B) = A^T A * B^T B
    A, B = signed_factors((13, 9, 1), 6, 61)[:2]
    H = O.hadamard(O.gram(A), O.gram(B))
    K = krp(A, B)
    assert np.allclose(H, K.T @ K, rtol=1e-13, atol=1e-13)
    assert np.array_equal(H, H.T)
    assert np.allclose(O.gram(A), A.T @ A, rtol=1e-14, atol=1e-14)


def test_norm_sq():
    T = random_tensor((7, 6, 5), 71, signed=True)
    assert abs(O.norm_sq(T) - math.fsum((T.ravel() ** 2).tolist())) <= 1e-14 * O.norm_sq(T)


def test_cholesky_and_solve_against_lapack():
    rng = np.random.default_rng(5)
    for R in (1, 2, 5, 20):
        A = rng.standard_normal((R + 3, R))
        H = A.T @ A
        rc, L = O.cholesky(H)
        assert rc == 0
        assert np.allclose(L, np.linalg.cholesky(H), rtol=1e-12, atol=1e-13)
        assert np.allclose(np.triu(L, 1), 0.0)
        b = rng.standard_normal(R)
        x = O.cholesky_solve(L, b)
        assert np.allclose(H @ x, b, rtol=0, atol=1e-10 * np.linalg.cond(H))
        assert np.allclose(x, np.linalg.solve(H, b), rtol=1e-9, atol=1e-12 * np.linalg.cond(H))


def test_cholesky_rejects_non_positive_definite():
    assert O.cholesky(np.array([[1.0, 2.0], [2.0, 1.0]]))[0] == 1
    assert O.cholesky(np.array([[0.0, 0.0], [0.0, 1.0]]))[0] == 1
    assert O.cholesky(np.array([[np.nan]]))[0] == 1
    assert O.cholesky(np.array([[np.inf]]))[0] == 1


# ------------------------------------------------------------------ one ALS iteration (Alg. 1)

def _lstsq_als_iteration(Tn, U):
    """One ALS sweep where every update is the plain linear least-squares problem
    min || T_(n)^T - KRP U_n^T ||, solved by LAPACK's SVD-based lstsq (not normal equations)."""
    U = [u.copy() for u in U]
    lam = None
    unf = [Tn.reshape(Tn.shape[0], -1), Tn.transpose(1, 0, 2).reshape(Tn.shape[1], -1),
           Tn.transpose(2, 0, 1).reshape(Tn.shape[2], -1)]
    for n in range(3):
        a, b = [m for m in range(3) if m != n]
        K = krp(U[a], U[b])
        X = np.linalg.lstsq(K, unf[n].T, rcond=None)[0].T
        lam = np.linalg.norm(X, axis=0)
        U[n] = X / lam
    return U, lam


def test_one_iteration_equals_three_least_squares_solves():
    dims, R = (10, 9, 8), 3
    T = random_tensor(dims, 81) + reconstruct(uniform_factors(dims, R, 82)).transpose(2, 1, 0)
    init = uniform_factors(dims, R, 83)
    m = O.Model(T, init, tol=-1.0, max_iters=5)
    U, lam = init, None
    for it in range(3):
        m.iterate()
        U, lam = _lstsq_als_iteration(tview(T), U)
        s = m.state()
        for n in range(3):
            assert np.allclose(s["U"][n], U[n], rtol=1e-9, atol=1e-11), (it, n)
        assert np.allclose(s["lam"], lam, rtol=1e-9)
        assert np.allclose(np.linalg.norm(s["U"][2], axis=0), 1.0, rtol=1e-14)


def test_fast_error_and_fit_equal_explicit_reconstruction():
    # Alg. 1, error line (sign of the middle term corrected): e = ||T - T_hat||^2.
    dims, R = (9, 7, 8), 4
    T = random_tensor(dims, 91)
    m = O.Model(T, uniform_factors(dims, R, 92), tol=-1.0, max_iters=20)
    nT = np.linalg.norm(T)
    for it in range(6):
        m.iterate()
        s = m.state()
        res = tview(T) - reconstruct(s["U"], s["lam"])
        e = float((res ** 2).sum())
        assert abs(s["err"] - e) <= 1e-12 * nT ** 2, it
        assert abs(s["fit"] - (1.0 - math.sqrt(e) / nT)) <= 1e-11, it


def test_error_never_increases_and_noise_free_tensor_is_recovered():
    dims, R = (20, 15, 10), 3
    true = uniform_factors(dims, R, 101)
    T = np.ascontiguousarray(reconstruct(true).transpose(2, 1, 0))
    r = O.cp_als(T, uniform_factors(dims, R, 102), tol=-1.0, max_iters=400)
    h = r["fit_history"]
    assert len(h) == 400
    # exact least squares per mode => the error cannot go up; near fit 1 the fast formula cancels
    # ||T||^2 against two terms of the same size, so the fit is only resolved to about sqrt(eps)
    far = h < 1.0 - 1e-4
    assert far.sum() > 5 and np.all(np.diff(h[far]) >= -1e-12)
    assert np.all(np.diff(h) >= -5e-8)
    assert 1.0 - h[-1] < 1e-6
    rel = np.linalg.norm(tview(T) - reconstruct(r["U"], r["lam"])) / np.linalg.norm(T)
    assert rel < 1e-7
    # factor congruence with the truth, up to permutation
    for n in range(3):
        tn = true[n] / np.linalg.norm(true[n], axis=0)
        Cg = np.abs(tn.T @ r["U"][n])
        assert np.all(Cg.max(axis=1) > 1 - 1e-6)


def test_rank_one_als_is_the_higher_order_power_method():
    dims = (8, 7, 6)
    T = random_tensor(dims, 111)
    Tn = tview(T)
    u = [x[:, 0].copy() for x in uniform_factors(dims, 1, 112)]
    m = O.Model(T, [x[:, None] for x in u], tol=-1.0, max_iters=10)
    lam = 1.0
    for it in range(4):
        m.iterate()
        # R = 1: H is the scalar (u_a.u_a)(u_b.u_b) and the update is the contraction divided by it
        v = np.einsum("ijk,j,k->i", Tn, u[1], u[2]) / ((u[1] @ u[1]) * (u[2] @ u[2]))
        u[0] = v / np.linalg.norm(v)
        v = np.einsum("ijk,i,k->j", Tn, u[0], u[2]) / ((u[0] @ u[0]) * (u[2] @ u[2]))
        u[1] = v / np.linalg.norm(v)
        v = np.einsum("ijk,i,j->k", Tn, u[0], u[1]) / ((u[0] @ u[0]) * (u[1] @ u[1]))
        lam = np.linalg.norm(v)
        u[2] = v / lam
        s = m.state()
        for n in range(3):
            assert np.allclose(s["U"][n][:, 0], u[n], rtol=1e-12, atol=1e-14)
        assert abs(s["lam"][0] - lam) <= 1e-12 * lam


def test_stop_rule_tolerance_and_iteration_cap():
    dims, R = (12, 11, 10), 3
    T = random_tensor(dims, 121) * 0.05 + reconstruct(uniform_factors(dims, R, 122)).transpose(2, 1, 0)
    init = uniform_factors(dims, R, 123)
    free = O.cp_als(T, init, tol=-1.0, max_iters=60)
    assert free["status"] == O.MAX_ITERS and free["iters"] == 60
    h = free["fit_history"]
    tol = float(np.sort(np.abs(np.diff(h)))[len(h) // 2])   # a tolerance this trajectory crosses midway
    first = next(i for i in range(1, len(h)) if abs(h[i] - h[i - 1]) < tol) + 1   # 1-based iteration
    stopped = O.cp_als(T, init, tol=tol, max_iters=60)
    assert stopped["status"] == O.CONVERGED and stopped["iters"] == first
    assert stopped["fit"] == h[first - 1]
    # "two consecutive iterations": never stops at iteration 1, even with a huge tolerance
    assert O.cp_als(T, init, tol=10.0, max_iters=60)["iters"] == 2
    assert O.cp_als(T, init, tol=10.0, max_iters=1)["status"] == O.MAX_ITERS


def test_cholesky_definite_uses_a_relative_pivot_test():
    rng = np.random.default_rng(7)
    A = rng.standard_normal((9, 5))
    H = A.T @ A
    rc, L = O.cholesky_definite(H)
    assert rc == 0 and np.allclose(L, np.linalg.cholesky(H), rtol=1e-12, atol=1e-13)
    B = np.hstack([A[:, :3], A[:, [1]], A[:, 3:]])             # a repeated column: exactly singular Gramian
    assert O.cholesky_definite(B.T @ B)[0] == 1
    assert O.cholesky_definite(np.diag([1.0, 0.0, 2.0]))[0] == 1
    for rel, want in [(1e-8, 0), (1e-10, 0), (1e-14, 1)]:       # second pivot = rel * its diagonal entry
        Hs = np.array([[1.0, np.sqrt(1.0 - rel)], [np.sqrt(1.0 - rel), 1.0]])
        assert O.cholesky_definite(Hs)[0] == want, rel
    assert O.cholesky_definite(np.array([[np.nan]]))[0] == 1


def test_pseudo_inverse_against_lapack_and_the_moore_penrose_conditions():
    rng = np.random.default_rng(8)
    for R, k in [(1, 1), (2, 1), (5, 3), (6, 6), (12, 7), (20, 19), (32, 16), (32, 32)]:
        A = rng.standard_normal((R, k)) * rng.uniform(0.1, 10.0, size=(1, k))
        H = A @ A.T
        H = 0.5 * (H + H.T)
        rc, P, rank = O.pinv_sym(H)
        assert rc == 0 and rank == k, (R, k, rank)
        want = np.linalg.pinv(H, rcond=O.RANK_TOL, hermitian=True)
        ev = np.linalg.eigvalsh(H)[::-1][:k]
        eps = 1e-14 * ev[0] / ev[-1]                              # rounding, amplified by the condition of the kept part
        scale = np.abs(want).max()
        assert np.abs(P - want).max() <= eps * scale, (R, k)
        nH = np.abs(H).max()
        assert np.abs(H @ P @ H - H).max() <= eps * nH
        assert np.abs(P @ H @ P - P).max() <= eps * scale
        assert np.abs(H @ P - (H @ P).T).max() <= eps and np.abs(P - P.T).max() <= 1e-13 * scale
    # structure: a zero row/column stays zero; a repeated row/column shares the weight equally
    H = np.array([[2.0, 0.0, 1.0], [0.0, 0.0, 0.0], [1.0, 0.0, 3.0]])
    rc, P, rank = O.pinv_sym(H)
    assert rc == 0 and rank == 2 and np.all(P[1] == 0.0) and np.all(P[:, 1] == 0.0)
    assert np.allclose(P[np.ix_([0, 2], [0, 2])], np.linalg.inv(H[np.ix_([0, 2], [0, 2])]), rtol=1e-13)
    rc, P, rank = O.pinv_sym(np.array([[4.0, 4.0], [4.0, 4.0]]))
    assert rc == 0 and rank == 1 and np.allclose(P, 1.0 / 16.0, rtol=1e-14)
    assert O.pinv_sym(np.zeros((3, 3)))[0] == 1
    assert O.pinv_sym(np.array([[1.0, np.inf], [np.inf, 1.0]]))[0] == 1


def _lstsq_min_norm_iteration(Tn, U):
    """One ALS sweep where every update is the MINIMUM-NORM least-squares solution of min ||T_(n)^T - K U_n^T||
    (LAPACK SVD; singular values of K below sqrt(RANK_TOL) of the largest count as zero)."""
    U = [u.copy() for u in U]
    lam = None
    for n in range(Tn.ndim):
        K = krp_all([U[m] for m in range(Tn.ndim) if m != n])
        X = np.linalg.lstsq(K, unfold(Tn, n).T, rcond=math.sqrt(O.RANK_TOL))[0].T
        lam = np.linalg.norm(X, axis=0)
        X[:, lam <= 1e-12 * lam.max()] = 0.0            # LAPACK leaves rounding dust where the exact answer is 0
        lam = np.linalg.norm(X, axis=0)
        U[n] = X / np.where(lam > 0, lam, 1.0)
    return U, lam


@pytest.mark.parametrize("kind", ["dead", "twin", "dead_and_twin"])
def test_rank_deficient_update_is_the_minimum_norm_solution_and_the_model_goes_on(kind):
    # Alg. 1, update line: U = M H^+.  A component that is zero in two modes (H has a zero row and column) and a
    # component that repeats another one (H has two equal rows and columns) make H exactly singular.
    dims, R = (7, 6, 5), 4
    T = random_tensor(dims, 131) + reconstruct(uniform_factors(dims, 2, 133)).transpose(2, 1, 0)
    init = uniform_factors(dims, R, 132)
    if "dead" in kind:
        init[1][:, 1] = 0.0
        init[2][:, 1] = 0.0
    if "twin" in kind:
        for n in range(3):
            init[n][:, 3] = init[n][:, 0]
    m = O.Model(T, init, tol=-1.0, max_iters=8)
    U, lam = init, None
    nT = np.linalg.norm(T)
    prev = None
    # (two identical components are an unstable arrangement: rounding differences between them grow about
    # sixty-fold per sweep until they separate, so that case is followed for four sweeps only)
    sweeps = 4 if "twin" in kind else 6
    for it in range(sweeps):
        assert m.iterate() == O.RUNNING
        U, lam = _lstsq_min_norm_iteration(tview(T), U)
        s = m.state()
        assert s["iters"] == it + 1
        if "twin" not in kind or it < 2:
            # (how two identical components share their weight is decided by rounding dust in the LAPACK route
            # after a few sweeps; their sum, checked below through the reconstruction, is not)
            for n in range(3):
                assert np.allclose(s["U"][n], U[n], rtol=1e-7, atol=1e-9), (it, n)
            assert np.allclose(s["lam"], lam, rtol=1e-7, atol=1e-9)
        assert np.allclose(reconstruct(s["U"], s["lam"]), reconstruct(U, lam), rtol=1e-7, atol=1e-9), it
        e = float(((tview(T) - reconstruct(s["U"], s["lam"])) ** 2).sum())
        assert abs(s["err"] - e) <= 1e-11 * nT ** 2 and abs(s["fit"] - (1 - math.sqrt(e) / nT)) <= 1e-10
        assert prev is None or e <= prev * (1 + 1e-12)
        prev = e
        if "dead" in kind:
            assert all(np.all(s["U"][n][:, 1] == 0.0) for n in range(3)) and s["lam"][1] == 0.0
        if "twin" in kind:
            assert all(np.allclose(s["U"][n][:, 3], s["U"][n][:, 0], rtol=1e-8, atol=1e-10) for n in range(3))
    # the same trajectory as the model without the redundant components (twins carry half the weight each)
    keep = [c for c in range(R) if not ("dead" in kind and c == 1) and not ("twin" in kind and c == 3)]
    small = O.cp_als(T, [u[:, keep] for u in init], tol=-1.0, max_iters=sweeps)
    s = m.state()
    assert abs(small["fit"] - s["fit"]) <= 1e-9
    assert np.allclose(reconstruct(small["U"], small["lam"]), reconstruct(s["U"], s["lam"]), rtol=1e-7, atol=1e-9)


def test_normal_equations_without_a_positive_eigenvalue_stop_the_model():
    dims, R = (6, 5, 4), 2
    T = random_tensor(dims, 131)
    init = uniform_factors(dims, R, 132)
    init[1][:] = 0.0                                            # H of the first update is the zero matrix
    r = O.cp_als(T, init, tol=-1.0, max_iters=5)
    assert r["status"] == O.NUMERICAL and r["iters"] == 0
    assert np.array_equal(r["U"][0], init[0])
    z = O.cp_als(np.zeros((4, 5, 6)), uniform_factors(dims, R, 132), tol=-1.0, max_iters=5)
    assert z["status"] == O.NUMERICAL and z["iters"] == 0       # all-zero tensor: the second update has H = 0


# ------------------------------------------------------------------ queue (Alg. 3)

def _read_schedules():
    out = []
    with open(os.path.join(GOLD, "queue_schedules.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [p.strip() for p in line.split(";")]
            ints = lambda s: [int(x) for x in s.split(",")]
            out.append((ints(parts[0]), ints(parts[1]), int(parts[2]), int(parts[3]), ints(parts[4]), ints(parts[5])))
    return out


@pytest.mark.parametrize("case", _read_schedules())
def test_queue_schedules_computed_by_hand(case):
    ranks, mits, rstar, slots, widths, order = case
    dims = (5, 4, 3)
    T = random_tensor(dims, 141)
    models = [dict(rank=r, init=uniform_factors(dims, r, 150 + k), tol=-1.0, max_iters=mi, flags=0, ls_alpha=1.0)
              for k, (r, mi) in enumerate(zip(ranks, mits))]
    out = O.cals(T, models, rstar, slots)
    assert list(out["total_rank_log"]) == widths
    assert list(out["retire_order"]) == order
    assert out["rounds"] == len(widths)
    assert list(out["iters"]) == mits


def test_golden_writer_steps_the_queue_like_the_oracle():
    # tests/golden/make_full_config_goldens.py steps Alg. 3 round by round over oracle.Model objects (to see every
    # iteration's fit); on a shrunken configuration 5 (line search, tolerance stops, 8 slots) its loop must give what
    # oracle.cals gives: order, rounds, iteration counts, statuses, fits -- bit for bit
    import importlib.util
    spec = importlib.util.spec_from_file_location("make_full_config_goldens", os.path.join(GOLD, "make_full_config_goldens.py"))
    G = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(G)
    from workloads import get_config, make_models, make_tensor
    cfg = get_config(5)
    dims = (40, 14, 13)
    T = make_tensor(cfg, dims=dims)
    models = make_models(cfg, dims=dims)[::4]
    for m in models:
        m["max_iters"] = 60
    rec, order, rounds, normT2 = G.lockstep(T, models, 60, 8, threads=2)
    ref = O.cals(T, models, 60, 8)
    assert order == list(ref["retire_order"]) and rounds == ref["rounds"] and normT2 == O.norm_sq(T)
    for k in range(len(models)):
        assert rec[k]["iters"] == ref["iters"][k] and rec[k]["status"] == ref["status"][k]
        assert rec[k]["fit"] == ref["fit"][k] and rec[k]["err"] == ref["err"][k]
        assert rec[k]["tol_margin"] >= 0.0 and len(rec[k]["fits"]) == rec[k]["iters"]
    # fixed iteration counts, everything resident: following a subset gives the same numbers and the same order
    cfg1 = get_config(1)
    T1 = make_tensor(cfg1)
    m1 = make_models(cfg1)
    for m in m1:
        m["max_iters"] = 5
    rec1, order1, rounds1, _ = G.lockstep(T1, m1, cfg1.max_total_rank, 0, threads=2, only={1, 7})
    ref1 = O.cals(T1, m1, cfg1.max_total_rank, 0)
    assert order1 == list(ref1["retire_order"]) and rounds1 == 5
    assert [k for k, r in enumerate(rec1) if r is not None] == [1, 7]
    assert rec1[7]["fit"] == ref1["fit"][7] and np.array_equal(rec1[7]["U"][0], ref1["U"][7][0])


def test_cals_results_do_not_depend_on_co_residents():
    # co-resident models do not influence each other (Sec. 1, contributions; Alg. 2): lock-step CALS == solo CP-ALS, bit for bit
    dims = (9, 8, 7)
    T = random_tensor(dims, 161) + reconstruct(uniform_factors(dims, 2, 162)).transpose(2, 1, 0)
    ranks = [1, 2, 3, 2, 4, 1]
    models = [dict(rank=r, init=uniform_factors(dims, r, 170 + k), tol=1e-4, max_iters=40, flags=0, ls_alpha=1.0)
              for k, r in enumerate(ranks)]
    a = O.cals(T, models, max_total_rank=sum(ranks))
    b = O.cals(T, models, max_total_rank=5, max_slots=2)
    for k, mdl in enumerate(models):
        solo = O.cp_als(T, mdl["init"], tol=1e-4, max_iters=40)
        for res in (a, b):
            assert res["iters"][k] == solo["iters"] and res["status"][k] == solo["status"]
            assert res["fit"][k] == solo["fit"]
            for n in range(3):
                assert np.array_equal(res["U"][k][n], solo["U"][n])
    assert sorted(a["retire_order"]) == list(range(len(ranks)))
    assert sorted(b["retire_order"]) == list(range(len(ranks)))
    # with everything resident the retirement order is (iteration count, slot)
    assert list(a["retire_order"]) == sorted(range(len(ranks)), key=lambda k: (a["iters"][k], k))
    with pytest.raises(ValueError):
        O.cals(T, models, max_total_rank=3)


# ------------------------------------------------------------------ non-negativity (Sec. 5)

def test_nnls_matches_lawson_hanson_library_and_kkt():
    rng = np.random.default_rng(7)
    for R in (1, 2, 3, 6, 12, 20):
        for trial in range(6):
            A = rng.standard_normal((R + 5, R))
            b = rng.standard_normal(R + 5) + 0.3
            H, m = A.T @ A, A.T @ b
            rc, x, P = O.nnls_row(H, m)
            assert rc == 0
            want, _ = scipy.optimize.nnls(A, b)
            assert np.allclose(x, want, rtol=1e-8, atol=1e-10)
            w = m - H @ x
            assert np.all(x >= 0)
            assert np.all(np.abs(w[x > 0]) <= 1e-9 * max(1.0, np.abs(m).max()))
            assert np.all(w[x == 0] <= 1e-9 * max(1.0, np.abs(m).max()))
            assert P == sum(1 << j for j in range(R) if x[j] > 0)
            # warm start from any set gives the same (unique) minimiser
            for warm in (P, (1 << R) - 1, 1):
                rc2, x2, _ = O.nnls_row(H, m, warm)
                assert rc2 == 0 and np.allclose(x2, x, rtol=1e-8, atol=1e-10)


def test_nnls_bounding_variable_leaves_the_passive_set():
    # right-hand sides (tests/golden/nnls_stall_cases.txt, written by make_nnls_stall_cases.py) on which a search
    # that removes passive variables only by "x <= 0 after the step" stalls at a non-optimal point: the variable
    # that bounds the step must leave the set even when rounding leaves it a tiny positive value
    lines = [ln for ln in open(os.path.join(GOLD, "nnls_stall_cases.txt")) if not ln.startswith("#")]
    H = np.array([float.fromhex(v) for v in lines[0].split()]).reshape(3, 3)
    rhs = [np.array([float.fromhex(v) for v in ln.split()]) for ln in lines[1:]]
    assert len(rhs) >= 20
    L = np.linalg.cholesky(H)
    for m in rhs:
        rc, x, P = O.nnls_row(H, m)
        want, _ = scipy.optimize.nnls(L.T, np.linalg.solve(L, m))
        f = lambda v: 0.5 * v @ H @ v - m @ v
        assert rc == 0 and x.min() >= 0.0
        assert f(x) <= f(want) + 1e-12 * abs(f(want))
        assert np.allclose(x, want, rtol=1e-7, atol=1e-9)
        w = m - H @ x                                   # KKT: gradient zero on the support, non-positive elsewhere
        assert np.all(np.abs(w[x > 0]) <= 1e-9 * np.abs(m).max()) and np.all(w[x == 0] <= 1e-9 * np.abs(m).max())
        assert P == sum(1 << j for j in range(3) if x[j] > 0)


def test_nnls_semidefinite_normal_equations_and_unusable_warm_start():
    # a dead component makes H only semi-definite (zero row and column): it must stay at zero, and a warm
    # start that contains it (so that its sub-block cannot be factorised) is dropped, not fatal
    rng = np.random.default_rng(9)
    R = 6
    A = rng.standard_normal((R + 4, R))
    A[:, 2] = 0.0
    b = rng.standard_normal(R + 4) + 0.5
    H, m = A.T @ A, A.T @ b
    want, _ = scipy.optimize.nnls(A, b)
    for warm in (0, 0b000100, 0b111111, 0b000101):
        rc, x, P = O.nnls_row(H, m, warm)
        assert rc == 0 and x[2] == 0.0 and not (P >> 2) & 1
        assert np.allclose(x, want, rtol=1e-8, atol=1e-10)
    # two identical columns: no unique minimiser; the search itself reaches a singular block -> reported
    A2 = rng.standard_normal((R + 4, R))
    A2[:, 1] = A2[:, 0]
    b2 = A2[:, 0] * 2.0 + 0.1
    rc, x, P = O.nnls_row(A2.T @ A2, A2.T @ b2, 0)
    assert rc in (0, 1)
    if rc == 0:   # then it is A minimiser: same objective value as the library's
        ref, _ = scipy.optimize.nnls(A2, b2)
        assert np.all(x >= 0) and abs(np.linalg.norm(A2 @ x - b2) - np.linalg.norm(A2 @ ref - b2)) < 1e-9


def test_nnls_brute_force_over_supports():
    rng = np.random.default_rng(8)
    R = 5
    for trial in range(10):
        A = rng.standard_normal((R + 2, R))
        b = rng.standard_normal(R + 2)
        H, m = A.T @ A, A.T @ b
        best, bestx = 0.0, np.zeros(R)
        for k in range(1, R + 1):
            for S in itertools.combinations(range(R), k):
                S = list(S)
                xs = np.linalg.solve(H[np.ix_(S, S)], m[S])
                if np.all(xs >= 0):
                    x = np.zeros(R)
                    x[S] = xs
                    f = 0.5 * x @ H @ x - m @ x
                    if f < best:
                        best, bestx = f, x
        rc, x, _ = O.nnls_row(H, m)
        assert rc == 0 and np.allclose(x, bestx, rtol=1e-8, atol=1e-10)


def test_nonneg_als_equals_plain_als_when_solution_is_positive_and_stays_nonneg_otherwise():
    dims, R = (10, 9, 8), 2
    true = uniform_factors(dims, R, 181)
    T = np.ascontiguousarray(reconstruct([t + 0.5 for t in true]).transpose(2, 1, 0))
    init = uniform_factors(dims, R, 182)
    near = [t + 0.5 + 0.05 * u for t, u in zip(true, init)]      # start close to the positive truth
    a = O.cp_als(T, near, tol=-1.0, max_iters=8)
    b = O.cp_als(T, near, tol=-1.0, max_iters=8, flags=O.FLAG_NONNEG)
    assert min(u.min() for u in a["U"]) > 0
    assert np.allclose(a["fit_history"], b["fit_history"], rtol=0, atol=1e-12)
    for n in range(3):
        assert np.allclose(a["U"][n], b["U"][n], rtol=1e-9, atol=1e-12)
    # a signed tensor: constrained factors stay >= 0, error still never increases, fast error still exact
    T2 = random_tensor(dims, 183, signed=True) + tview(T).transpose(2, 1, 0) * 0.3
    T2 = np.ascontiguousarray(T2)
    m = O.Model(T2, init, tol=-1.0, max_iters=30, flags=O.FLAG_NONNEG)
    prev = None
    for it in range(12):
        m.iterate()
        s = m.state()
        assert min(u.min() for u in s["U"]) >= 0.0
        e = float(((tview(T2) - reconstruct(s["U"], s["lam"])) ** 2).sum())
        assert abs(e - s["err"]) <= 1e-11 * np.linalg.norm(T2) ** 2
        if prev is not None:
            assert s["err"] <= prev + 1e-10
        prev = s["err"]
    unc = O.cp_als(T2, init, tol=-1.0, max_iters=12)
    assert min(u.min() for u in unc["U"]) < 0   # the constraint was active in this problem


# ------------------------------------------------------------------ line search (Sec. 5)

def test_line_search_accepts_only_improvements_and_error_stays_exact():
    dims, R = (14, 12, 10), 3
    # collinear truth => slow ALS convergence, where extrapolation is worth something
    base = uniform_factors(dims, 1, 191)
    true = [np.hstack([b + 0.15 * u[:, [r]] for r in range(R)]) for b, u in zip(base, uniform_factors(dims, R, 192))]
    T = np.ascontiguousarray(reconstruct(true).transpose(2, 1, 0)) + 0.001 * random_tensor(dims, 193, signed=True)
    init = uniform_factors(dims, R, 194)
    m = O.Model(T, init, tol=-1.0, max_iters=200, flags=O.FLAG_LINESEARCH, alpha=1.3)
    plain = O.Model(T, init, tol=-1.0, max_iters=200)
    nT2 = np.linalg.norm(T) ** 2
    prev, acc_prev = None, 0
    for it in range(40):
        m.iterate()
        plain.iterate()
        s = m.state()
        e = float(((tview(T) - reconstruct(s["U"], s["lam"])) ** 2).sum())
        assert abs(e - s["err"]) <= 1e-11 * nT2, it
        if prev is not None:
            assert s["err"] <= prev * (1 + 1e-12)
        if it == 0:
            assert s["ls_accepted"] == 0 and s["err"] == plain.state()["err"]   # nothing to extrapolate from yet
        if s["ls_accepted"] > acc_prev:
            assert np.array_equal(s["lam"], np.ones(R))          # accepted point carries lambda = 1
        prev, acc_prev = s["err"], s["ls_accepted"]
    assert acc_prev > 0
    assert m.state()["err"] < plain.state()["err"]               # and it did help on this problem


def test_line_search_with_alpha_one_changes_nothing_material():
    dims, R = (8, 7, 6), 2
    T = random_tensor(dims, 201)
    init = uniform_factors(dims, R, 202)
    a = O.cp_als(T, init, tol=-1.0, max_iters=15)
    b = O.cp_als(T, init, tol=-1.0, max_iters=15, flags=O.FLAG_LINESEARCH, alpha=1.0)
    assert np.allclose(a["fit_history"], b["fit_history"], rtol=0, atol=1e-13)



# ------------------------------------------------------------------ non-negativity with line search together

def _nn_ls_problem():
    dims, R = (12, 10, 9), 3
    base = uniform_factors(dims, 1, 401)
    true = [np.hstack([b + 0.2 * u[:, [r]] for r in range(R)]) for b, u in zip(base, uniform_factors(dims, R, 402))]
    T = np.ascontiguousarray(reconstruct(true).transpose(2, 1, 0)) + 0.05 * random_tensor(dims, 403, signed=True)
    return dims, R, T, uniform_factors(dims, R, 404)


def test_nonneg_line_search_visits_only_feasible_points_and_keeps_the_error_exact():
    dims, R, T, init = _nn_ls_problem()
    both = O.FLAG_NONNEG | O.FLAG_LINESEARCH
    m = O.Model(T, init, tol=-1.0, max_iters=100, flags=both, alpha=1.6)
    nT2 = np.linalg.norm(T) ** 2
    prev = None
    for it in range(40):
        m.iterate()
        s = m.state()
        assert min(u.min() for u in s["U"]) >= 0.0 and s["lam"].min() >= 0.0
        e = float(((tview(T) - reconstruct(s["U"], s["lam"])) ** 2).sum())
        assert abs(e - s["err"]) <= 1e-11 * nT2, it
        if prev is not None:
            assert s["err"] <= prev * (1 + 1e-12) + 1e-12 * nT2
        prev = s["err"]
    assert m.state()["ls_accepted"] > 0
    # alpha = 1: the "extrapolated" point is the current one, never strictly better: the NONNEG run, unchanged
    a = O.cp_als(T, init, tol=-1.0, max_iters=15, flags=O.FLAG_NONNEG)
    b = O.cp_als(T, init, tol=-1.0, max_iters=15, flags=both, alpha=1.0)
    assert np.allclose(a["fit_history"], b["fit_history"], rtol=0, atol=1e-13)


def test_nonneg_line_search_steps_replayed_by_hand_with_clipping():
    # every iteration of a NONNEG+LINESEARCH model rebuilt from a NONNEG-only iteration and numpy: from the point
    # kept so far (lambda folded into mode 3) a fresh NONNEG model gives the ALS point; the candidate is
    # max(0, P_prev + alpha (P_als - P_prev)) entry by entry, taken iff its explicit residual is smaller
    dims, R, T, init = _nn_ls_problem()
    alpha = 2.5                                   # far enough for some entries to cross zero
    err = lambda P: float(((tview(T) - reconstruct(P)) ** 2).sum())
    point = lambda st: [st["U"][0], st["U"][1], st["U"][2] * st["lam"]]
    m = O.Model(T, init, tol=-1.0, max_iters=60, flags=O.FLAG_NONNEG | O.FLAG_LINESEARCH, alpha=alpha)
    m.iterate()
    assert m.state()["ls_accepted"] == 0          # nothing to extrapolate from after the first iteration
    taken_clipped = rejected = 0
    for it in range(2, 14):
        before = m.state()
        P_prev = point(before)
        fresh = O.Model(T, P_prev, tol=-1.0, max_iters=5, flags=O.FLAG_NONNEG)
        fresh.iterate()
        P_als = point(fresh.state())
        raw = [a + alpha * (b - a) for a, b in zip(P_prev, P_als)]
        cand = [np.maximum(x, 0.0) for x in raw]
        e_als, e_cand = err(P_als), err(cand)
        m.iterate()
        after = m.state()
        take = e_cand < e_als
        assert after["ls_accepted"] - before["ls_accepted"] == int(take), it
        want = cand if take else P_als
        for n in range(3):
            assert np.allclose(point(after)[n], want[n], rtol=1e-9, atol=1e-11), (it, n)
        assert abs(after["err"] - (e_cand if take else e_als)) <= 1e-11 * np.linalg.norm(T) ** 2
        taken_clipped += int(take and min(x.min() for x in raw) < 0.0)
        rejected += int(not take)
    assert taken_clipped > 0 and rejected > 0     # both branches, and the projection mattered in an accepted step


# ------------------------------------------------------------------ order-N tensors (Alg. 1 for N modes)

def nview(T):
    """numpy view of an order-N tensor indexed [i1, ..., iN]."""
    return T.transpose(*range(T.ndim - 1, -1, -1))


def reconstruct_nd(U, lam=None):
    lam = np.ones(U[0].shape[1]) if lam is None else lam
    out = lam[None, :] * U[0]
    for u in U[1:]:
        out = out[..., None, :] * u
    return out.sum(axis=-1)


def krp_all(mats):
    """Khatri-Rao product of a list, first matrix's row index slowest."""
    K = mats[0]
    for B in mats[1:]:
        K = krp(K, B)
    return K


def unfold(Tn, n):
    """Mode-n unfolding with the remaining indices in increasing mode order, the first of them slowest."""
    return np.moveaxis(Tn, n, 0).reshape(Tn.shape[n], -1)


@pytest.mark.parametrize("dims", [(3, 4, 2, 3), (2, 3, 2, 2, 3), (2, 1, 3, 2), (2, 2, 2, 2, 2, 2)])
def test_mttkrp_nd_brute_force_loops(dims):
    R, N = 2, len(dims)
    T = random_tensor(dims, 211, signed=True)
    U = signed_factors(dims, R, 212)
    Tn = nview(T)
    want = [np.zeros((d, R)) for d in dims]
    for idx in itertools.product(*[range(d) for d in dims]):
        for r in range(R):
            for n in range(N):
                k = 1.0
                for m in range(N):
                    if m != n:
                        k *= U[m][idx[m], r]
                want[n][idx[n], r] += Tn[idx] * k
    for mode in range(1, N + 1):
        got = O.mttkrp(T, U, mode)
        assert np.allclose(got, want[mode - 1], rtol=1e-13, atol=1e-14), mode


def test_mttkrp_nd_is_unfolding_times_explicit_krp_and_matches_einsum():
    dims, R = (7, 5, 6, 4), 5
    T = random_tensor(dims, 221, signed=True)
    U = signed_factors(dims, R, 222)
    Tn = nview(T)
    ein = ["jr,kr,lr,ijkl->ir", "ir,kr,lr,ijkl->jr", "ir,jr,lr,ijkl->kr", "ir,jr,kr,ijkl->lr"]
    for n in range(4):
        others = [U[m] for m in range(4) if m != n]
        want = unfold(Tn, n) @ krp_all(others)
        got = O.mttkrp(T, U, n + 1)
        scale = np.abs(want).max()
        assert np.abs(got - want).max() <= 1e-12 * scale, n
        assert np.abs(got - np.einsum(ein[n], *others, Tn)).max() <= 1e-12 * scale, n


def test_mttkrp_nd_fused_columns_equal_solo_results_bitwise_and_element_is_the_exact_sum():
    dims = (4, 3, 5, 3)
    T = random_tensor(dims, 231, signed=True)
    ranks = [1, 3, 2, 9]
    facs = [signed_factors(dims, r, 232 + k) for k, r in enumerate(ranks)]
    fused = [np.hstack([f[n] for f in facs]) for n in range(4)]
    Tn = nview(T)
    for mode in range(1, 5):
        big = O.mttkrp(T, fused, mode)
        c = 0
        for f, r in zip(facs, ranks):
            assert np.array_equal(big[:, c:c + r], O.mttkrp(T, f, mode)), (mode, r)
            c += r
    for mode, row, col in [(1, 3, 2), (2, 0, 14), (3, 4, 7), (4, 2, 0)]:
        terms = []
        for idx in itertools.product(*[range(d) for d in dims]):
            if idx[mode - 1] != row:
                continue
            k = 1.0
            for m in range(4):
                if m != mode - 1:
                    k *= fused[m][idx[m], col]
            terms.append(Tn[idx] * k)
        v, sa = O.mttkrp_element(T, fused, mode, row, col)
        assert abs(v - math.fsum(terms)) <= 4e-16 * math.fsum(abs(t) for t in terms)
        assert abs(sa - math.fsum(abs(t) for t in terms)) <= 1e-15 * sa
        assert abs(O.mttkrp(T, fused, mode)[row, col] - v) <= 1e-14 * sa


def test_norm_sq_nd():
    T = random_tensor((4, 3, 5, 2, 3), 241, signed=True)
    assert abs(O.norm_sq(T) - math.fsum((T.ravel() ** 2).tolist())) <= 1e-14 * O.norm_sq(T)


@pytest.mark.parametrize("where", [0, 1, 2, 3])
@pytest.mark.parametrize("flags,alpha", [(0, 1.0), (O.FLAG_NONNEG, 1.0), (O.FLAG_LINESEARCH, 1.25)])
def test_order_4_with_a_singleton_mode_is_the_order_3_problem(where, flags, alpha):
    # a mode of extent 1 whose factor is the 1 x R matrix of ones contributes factors of exactly 1 everywhere
    if where == 3 and flags & O.FLAG_LINESEARCH:
        # line search moves each factor matrix along a straight line, with lambda folded into the LAST mode's
        # factor: a trailing singleton takes lambda away from mode 3, which is a different (equally valid) path
        pytest.skip("extrapolation is not invariant to where the column scales are kept")
    dims3, R = (6, 5, 4), 3
    T3 = random_tensor(dims3, 251) + reconstruct(uniform_factors(dims3, R, 252)).transpose(2, 1, 0)
    init3 = uniform_factors(dims3, R, 253)
    dims4 = list(dims3)
    dims4.insert(where, 1)
    shape4 = tuple(dims4)[::-1]
    T4 = np.ascontiguousarray(T3.reshape(shape4))
    init4 = list(init3)
    init4.insert(where, np.ones((1, R)))
    a = O.Model(T3, init3, tol=-1.0, max_iters=8, flags=flags, alpha=alpha)
    b = O.Model(T4, init4, tol=-1.0, max_iters=8, flags=flags, alpha=alpha)
    for it in range(6):
        a.iterate()
        b.iterate()
        sa, sb = a.state(), b.state()
        full3 = reconstruct(sa["U"], sa["lam"])
        full4 = reconstruct_nd(sb["U"], sb["lam"]).reshape(full3.shape)
        assert np.allclose(full3, full4, rtol=1e-9, atol=1e-11), it
        assert abs(sa["fit"] - sb["fit"]) <= 1e-11, it
        assert abs(sa["err"] - sb["err"]) <= 1e-10 * O.norm_sq(T3), it
        assert sa["ls_accepted"] == sb["ls_accepted"]
        if flags & O.FLAG_NONNEG:
            assert min(u.min() for u in sb["U"]) >= 0.0


def _lstsq_als_iteration_nd(Tn, U):
    U = [u.copy() for u in U]
    lam = None
    for n in range(Tn.ndim):
        K = krp_all([U[m] for m in range(Tn.ndim) if m != n])
        X = np.linalg.lstsq(K, unfold(Tn, n).T, rcond=None)[0].T
        lam = np.linalg.norm(X, axis=0)
        U[n] = X / lam
    return U, lam


@pytest.mark.parametrize("dims", [(7, 6, 5, 4), (4, 3, 5, 3, 4)])
def test_nd_iteration_equals_least_squares_solves_and_fast_error_is_the_residual(dims):
    R = 3
    T = low_rank_tensor(dims, R, 261, noise=0.3)
    init = uniform_factors(dims, R, 262)
    m = O.Model(T, init, tol=-1.0, max_iters=5)
    U, lam = init, None
    nT = np.linalg.norm(T)
    for it in range(3):
        m.iterate()
        U, lam = _lstsq_als_iteration_nd(nview(T), U)
        s = m.state()
        for n in range(len(dims)):
            assert np.allclose(s["U"][n], U[n], rtol=1e-8, atol=1e-10), (it, n)
        assert np.allclose(s["lam"], lam, rtol=1e-8)
        e = float(((nview(T) - reconstruct_nd(s["U"], s["lam"])) ** 2).sum())
        assert abs(s["err"] - e) <= 1e-12 * nT ** 2, it
        assert abs(s["fit"] - (1.0 - math.sqrt(e) / nT)) <= 1e-11, it


def test_nd_noise_free_tensor_is_recovered_and_error_never_increases():
    dims, R = (8, 7, 6, 5), 2
    T = low_rank_tensor(dims, R, 271)
    r = O.cp_als(T, uniform_factors(dims, R, 272), tol=-1.0, max_iters=300)
    h = r["fit_history"]
    far = h < 1.0 - 1e-4
    assert np.all(np.diff(h[far]) >= -1e-12) and np.all(np.diff(h) >= -5e-8)
    assert 1.0 - h[-1] < 1e-6
    rel = np.linalg.norm(nview(T) - reconstruct_nd(r["U"], r["lam"])) / np.linalg.norm(T)
    assert rel < 1e-6


def test_nd_line_search_accepts_only_improvements_and_error_stays_exact():
    dims, R = (7, 6, 5, 4), 3
    base = uniform_factors(dims, 1, 281)
    true = [np.hstack([b + 0.15 * u[:, [r]] for r in range(R)]) for b, u in zip(base, uniform_factors(dims, R, 282))]
    T = np.ascontiguousarray(reconstruct_nd(true).transpose(3, 2, 1, 0)) + 0.001 * random_tensor(dims, 283, signed=True)
    init = uniform_factors(dims, R, 284)
    m = O.Model(T, init, tol=-1.0, max_iters=200, flags=O.FLAG_LINESEARCH, alpha=1.3)
    nT2 = np.linalg.norm(T) ** 2
    prev, acc_prev = None, 0
    for it in range(40):
        m.iterate()
        s = m.state()
        e = float(((nview(T) - reconstruct_nd(s["U"], s["lam"])) ** 2).sum())
        assert abs(e - s["err"]) <= 1e-11 * nT2, it
        if prev is not None:
            assert s["err"] <= prev * (1 + 1e-12)
        if s["ls_accepted"] > acc_prev:
            assert np.array_equal(s["lam"], np.ones(R))
        prev, acc_prev = s["err"], s["ls_accepted"]
    assert acc_prev > 0


def test_nd_cals_results_do_not_depend_on_co_residents():
    dims = (5, 4, 3, 4)
    T = low_rank_tensor(dims, 2, 291, noise=0.5)
    ranks = [1, 2, 3, 2, 4, 1]
    models = [dict(rank=r, init=uniform_factors(dims, r, 300 + k), tol=1e-4, max_iters=40, flags=0, ls_alpha=1.0)
              for k, r in enumerate(ranks)]
    a = O.cals(T, models, max_total_rank=sum(ranks))
    b = O.cals(T, models, max_total_rank=5, max_slots=2)
    for k, mdl in enumerate(models):
        solo = O.cp_als(T, mdl["init"], tol=1e-4, max_iters=40)
        for res in (a, b):
            assert res["iters"][k] == solo["iters"] and res["status"][k] == solo["status"]
            assert res["fit"][k] == solo["fit"]
            for n in range(4):
                assert np.array_equal(res["U"][k][n], solo["U"][n])
    assert list(a["retire_order"]) == sorted(range(len(ranks)), key=lambda k: (a["iters"][k], k))
    assert sorted(b["retire_order"]) == list(range(len(ranks)))


def test_nd_mttkrp_of_modes_2_to_N_factors_through_the_mode_1_contraction():
    # the identity behind two-step sweeps for any order: with Y[i2..iN, c] = sum_i1 T U1, the MTTKRP of mode n >= 2
    # is Y contracted with the factors of the remaining modes, column by column
    dims, R = (5, 4, 6, 3, 4), 3
    T = random_tensor(dims, 501, signed=True)
    U = signed_factors(dims, R, 502)
    Y = np.einsum("ijklm,ir->jklmr", nview(T), U[0])
    want = {2: np.einsum("jklmr,kr,lr,mr->jr", Y, U[2], U[3], U[4]), 3: np.einsum("jklmr,jr,lr,mr->kr", Y, U[1], U[3], U[4]),
            4: np.einsum("jklmr,jr,kr,mr->lr", Y, U[1], U[2], U[4]), 5: np.einsum("jklmr,jr,kr,lr->mr", Y, U[1], U[2], U[3])}
    for mode, w in want.items():
        got = O.mttkrp(T, U, mode)
        assert np.abs(got - w).max() <= 1e-12 * np.abs(w).max(), mode
