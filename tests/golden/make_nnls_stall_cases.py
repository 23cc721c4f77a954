"""Writes tests/golden/nnls_stall_cases.txt: a normal-equation matrix H and right-hand sides on which an active-set
search that takes variables out of the passive set only by the test "x <= 0 after the step" stalls: the variable
that bounds the step comes out of x + beta (s - x) as a tiny positive number instead of zero, stays passive, and
the search creeps (shrinking that number sixteen digits per step) until its step cap, far from the minimiser.

The cases are rows of the first non-negative ALS iteration on a 20 x 30 x 100003 tensor (mode 3; H = Hadamard
product of the Gramians of the freshly updated, nearly collinear mode-1 and mode-2 factors).  They are found here
with `flawed_search`, a transcription of the search with that removal rule.  Everything comes from the seeded
generators, the CPU oracle and this file; expected solutions are NOT stored (the test asks scipy).
Run from the repository root:  python tests/golden/make_nnls_stall_cases.py
"""
import math
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle as O  # noqa: E402
from workloads import random_tensor, uniform_factors  # noqa: E402


def _chol_solve(H, idx, m):
    n = len(idx)
    L = [[0.0] * n for _ in range(n)]
    for j in range(n):
        d = H[idx[j]][idx[j]]
        for k in range(j):
            d -= L[j][k] * L[j][k]
        if not d > 0.0:
            return None
        d = math.sqrt(d)
        L[j][j] = d
        for i in range(j + 1, n):
            v = H[idx[i]][idx[j]]
            for k in range(j):
                v -= L[i][k] * L[j][k]
            L[i][j] = v / d
    x = [m[i] for i in idx]
    for i in range(n):
        v = x[i]
        for k in range(i):
            v -= L[i][k] * x[k]
        x[i] = v / L[i][i]
    for i in range(n - 1, -1, -1):
        v = x[i]
        for k in range(i + 1, n):
            v -= L[k][i] * x[k]
        x[i] = v / L[i][i]
    return x


def flawed_search(H, m):
    """Lawson-Hanson on (H, m) from the empty set, removal by "x <= 0" only.  Returns True if it hits the step cap."""
    R = len(m)
    tau = 10.0 * sys.float_info.epsilon * max(sum(abs(H[i][j]) for i in range(R)) for j in range(R)) * R
    cap, steps = 30 * R, 0
    P, x = [], [0.0] * R
    while True:
        while P:
            idx = sorted(P)
            s = _chol_solve(H, idx, m)
            if s is None:
                return False
            if all(v > 0.0 for v in s):
                x = [0.0] * R
                for a, j in enumerate(idx):
                    x[j] = s[a]
                break
            beta = 1.0
            for a, j in enumerate(idx):
                if not s[a] > 0.0:
                    q = x[j] / (x[j] - s[a]) if x[j] != s[a] else float("nan")
                    if q < beta:
                        beta = q
            for a, j in enumerate(idx):
                x[j] = x[j] + beta * (s[a] - x[j])
                if not x[j] > 0.0:
                    x[j] = 0.0
                    P.remove(j)
            steps += 1
            if steps > cap:
                return True
        best, wbest = -1, tau
        for j in range(R):
            if j in P:
                continue
            w = m[j]
            for k in range(R):
                w -= H[j][k] * x[k]
            if w > wbest:
                wbest, best = w, j
        if best < 0:
            return False
        P.append(best)
        steps += 1
        if steps > cap:
            return True


def main():
    dims = (20, 30, 100003)
    A = uniform_factors(dims, 3, 4100)
    T = np.einsum("ir,jr,kr->kji", *A)
    T = np.ascontiguousarray(T + 0.1 * random_tensor(dims, 4101, signed=True) * np.sqrt((T ** 2).mean()))
    U = [u.copy() for u in uniform_factors(dims, 3, 4303)]
    for n in (0, 1):                                   # the first two mode updates of a NONNEG iteration
        a, b = [k for k in range(3) if k != n]
        H = O.hadamard(O.gram(U[a]), O.gram(U[b]))
        M = O.mttkrp(T, U, n + 1)
        X = np.array([O.nnls_row(H, M[i])[1] for i in range(M.shape[0])])
        U[n] = X / np.linalg.norm(X, axis=0)
    H = np.asarray(O.hadamard(O.gram(U[0]), O.gram(U[1])))
    M = O.mttkrp(T, U, 3)
    Hl = [[float(v) for v in row] for row in H]
    rows = [i for i in range(M.shape[0]) if flawed_search(Hl, [float(v) for v in M[i]])]
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "nnls_stall_cases.txt")
    with open(out, "w") as f:
        f.write("# written by tests/golden/make_nnls_stall_cases.py; hexadecimal doubles\n")
        f.write("# first line: the 3 x 3 matrix H row by row; then one right-hand side per line (%d cases)\n" % len(rows))
        f.write(" ".join(float(v).hex() for v in H.ravel()) + "\n")
        for i in rows:
            f.write(" ".join(float(v).hex() for v in M[i]) + "\n")
    print("wrote", out, len(rows), "cases")


if __name__ == "__main__":
    main()
