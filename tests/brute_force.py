"""Exhaustive solvers used only to pin the oracle's ISTA on tiny problems.

They reach the answers by enumeration, not by iteration, so they share no
failure mode with the decoder they check.
"""
import itertools

import numpy as np


def l0_support_search(Phi, y, k):
    """Support of size k whose least-squares fit has the smallest residual (all C(n,k) tried)."""
    n = Phi.shape[1]
    best, best_res = None, np.inf
    for sup in itertools.combinations(range(n), k):
        cols = Phi[:, sup]
        coef, *_ = np.linalg.lstsq(cols, y, rcond=None)
        res = np.linalg.norm(y - cols @ coef)
        if res < best_res:
            best, best_res = sup, res
    return np.array(best), best_res


def lasso_by_kkt_enumeration(Phi, y, lam, tol=1e-10):
    """Exact minimiser of 1/2||y - Phi x||^2 + lam ||x||_1 by trying every (support, sign)
    pattern and keeping the one that satisfies the optimality (KKT) conditions:
      on the support   Phi_S^T (y - Phi x) = lam * sign(x_S)
      off the support  |Phi_j^T (y - Phi x)| <= lam.
    Returns x or None if no pattern passes (degenerate problem)."""
    m, n = Phi.shape
    for size in range(0, min(m, n) + 1):
        for sup in itertools.combinations(range(n), size):
            sup = list(sup)
            for signs in itertools.product((-1.0, 1.0), repeat=size):
                x = np.zeros(n)
                if size:
                    A = Phi[:, sup]
                    G = A.T @ A
                    if np.linalg.cond(G) > 1e12:
                        continue
                    xs = np.linalg.solve(G, A.T @ y - lam * np.array(signs))
                    if np.any(np.sign(xs) != np.array(signs)):
                        continue
                    x[sup] = xs
                corr = Phi.T @ (y - Phi @ x)
                off = np.setdiff1d(np.arange(n), sup)
                if np.all(np.abs(corr[off]) <= lam + tol):
                    return x
    return None
