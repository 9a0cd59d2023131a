"""Exact-optimum checker for tiny instances -- test infrastructure only.

A dense two-phase tableau simplex with Bland's anti-cycling rule, and the path-form LP of the
planner's problem (Eq. (1)-(5) of Sec. IV-B, relaxed to fractions and capacity-normalized):

    minimise lambda
    s.t.  sum_{p in paths(k)} x_p = 1                      for every commodity k
          sum_{p through e} (d_k(p)/cap_e) x_p <= lambda   for every link e
          x >= 0, lambda >= 0

Used only to pin the oracle's lambda within the multiplicative-weights guarantee on inputs small
enough for a brute-force solver.
"""
from __future__ import annotations

import numpy as np


def simplex_standard(c, A, b, tol=1e-11, max_pivots=200000):
    """min c.x  s.t.  A x = b, x >= 0, with b >= 0.  Returns (objective, x)."""
    A = np.array(A, dtype=np.float64)
    b = np.array(b, dtype=np.float64)
    c = np.array(c, dtype=np.float64)
    m, n = A.shape
    if np.any(b < 0):
        raise ValueError("b must be non-negative")
    # phase I: artificial variables n..n+m-1 form the first basis
    T = np.zeros((m + 1, n + m + 1))
    T[:m, :n] = A
    T[:m, n:n + m] = np.eye(m)
    T[:m, -1] = b
    basis = list(range(n, n + m))
    cost1 = np.concatenate([np.zeros(n), np.ones(m)])

    def set_objective(cost):
        T[m, :] = 0.0
        T[m, :len(cost)] = cost
        for r, j in enumerate(basis):
            if T[m, j] != 0.0:
                T[m, :] -= T[m, j] * T[r, :]

    def run(ncols):
        for _ in range(max_pivots):
            col = -1
            for j in range(ncols):              # Bland: lowest index with negative reduced cost
                if T[m, j] < -tol:
                    col = j
                    break
            if col < 0:
                return
            best, row = None, -1
            for r in range(m):
                a = T[r, col]
                if a > tol:
                    ratio = T[r, -1] / a
                    if (best is None or ratio < best - 1e-15 or
                            (abs(ratio - best) <= 1e-15 and basis[r] < basis[row])):
                        best, row = ratio, r
            if row < 0:
                raise ArithmeticError("LP unbounded")
            T[row, :] /= T[row, col]
            for r in range(m + 1):
                if r != row and T[r, col] != 0.0:
                    T[r, :] -= T[r, col] * T[row, :]
            basis[row] = col
        raise ArithmeticError("simplex did not terminate")

    set_objective(cost1)
    run(n + m)
    if -T[m, -1] > 1e-8:
        raise ArithmeticError("LP infeasible")
    # drive remaining artificial variables out of the basis where possible
    for r in range(m):
        if basis[r] >= n:
            for j in range(n):
                if abs(T[r, j]) > tol:
                    T[r, :] /= T[r, j]
                    for rr in range(m + 1):
                        if rr != r and T[rr, j] != 0.0:
                            T[rr, :] -= T[rr, j] * T[r, :]
                    basis[r] = j
                    break
    T[:, n:n + m] = 0.0                          # artificials may not re-enter
    set_objective(c)
    run(n)
    x = np.zeros(n)
    for r, j in enumerate(basis):
        if j < n:
            x[j] = T[r, -1]
    return float(c @ x), x


def min_congestion_lp(n_links, cap, comm_path_ptr, path_link_ptr, path_links, demand):
    """Builds and solves the LP above.  Returns (lambda_opt, splits)."""
    cp = np.asarray(comm_path_ptr)
    lp = np.asarray(path_link_ptr)
    pl = np.asarray(path_links)
    K, P, E = len(cp) - 1, len(lp) - 1, int(n_links)
    d = np.asarray(demand, dtype=np.float64)
    cap = np.asarray(cap, dtype=np.float64)
    util = np.zeros((E, P))
    for k in range(K):
        for p in range(cp[k], cp[k + 1]):
            for i in range(lp[p], lp[p + 1]):
                util[pl[i], p] += d[k] / cap[pl[i]]
    scale = util.max() if util.max() > 0 else 1.0
    util /= scale
    # variables: x_0..x_{P-1}, lambda, slack_0..slack_{E-1}
    n = P + 1 + E
    A = np.zeros((K + E, n))
    b = np.zeros(K + E)
    for k in range(K):
        A[k, cp[k]:cp[k + 1]] = 1.0
        b[k] = 1.0
    A[K:, :P] = util
    A[K:, P] = -1.0
    A[K:, P + 1:] = np.eye(E)
    c = np.zeros(n)
    c[P] = 1.0
    obj, x = simplex_standard(c, A, b)
    return obj * scale, x[:P]
