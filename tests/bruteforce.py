"""Independent ground truth for tiny instances, used only to pin the oracle.

Nothing here follows the oracle's route: objectives are written from A, alpha and the labels
directly (never from a running shared vector), and optima come from enumerating the KKT
systems of all active sets with numpy's dense solvers.
"""
import itertools

import numpy as np


def lasso_objective(A, b, alpha, lam):
    """||A alpha - b||^2/(2d) + lam ||alpha||_1 with A given as a plain d x n matrix."""
    d = A.shape[0]
    r = A @ alpha - b
    return float(r @ r) / (2 * d) + lam * float(np.abs(alpha).sum())


def svm_dual_objective(A, y, alpha, lam):
    """-(1/n) sum y_i alpha_i + ||A alpha||^2 / (2 lam n^2)."""
    n = A.shape[1]
    u = A @ alpha
    return -float(y @ alpha) / n + float(u @ u) / (2 * lam * n * n)


def svm_primal_objective(A, y, w, lam):
    """(1/n) sum max(0, 1 - y_i a_i^T w) + lam/2 ||w||^2."""
    n = A.shape[1]
    return float(np.maximum(0.0, 1.0 - y * (A.T @ w)).sum()) / n + 0.5 * lam * float(w @ w)


def enet_objective(A, b, alpha, lam, eta):
    """||A alpha - b||^2/(2d) + lam (eta/2 ||alpha||^2 + (1-eta) ||alpha||_1)."""
    d = A.shape[0]
    r = A @ alpha - b
    return float(r @ r) / (2 * d) + lam * (0.5 * eta * float(alpha @ alpha) + (1 - eta) * float(np.abs(alpha).sum()))


def enet_gap(A, b, alpha, lam, eta):
    """Total duality gap of Section 2, eq. (2), from the conjugates written out: f(u) =
    ||u - b||^2/(2d), f*(w) = w^T b + (d/2)||w||^2, g_i*(u) = [|u| - lam(1-eta)]_+^2/(2 lam eta),
    at w = grad f(A alpha)."""
    d = A.shape[0]
    w = (A @ alpha - b) / d
    u = -(A.T @ w)
    gstar = np.maximum(np.abs(u) - lam * (1 - eta), 0.0) ** 2 / (2 * lam * eta)
    return enet_objective(A, b, alpha, lam, eta) + float(w @ b) + 0.5 * d * float(w @ w) + float(gstar.sum())


def enet_optimum(A, b, lam, eta):
    """Exact elastic-net minimiser by enumerating sign patterns (n <= ~8); eta = 1 has the single
    pattern-free solution of the ridge normal equations."""
    d, n = A.shape
    best = (enet_objective(A, b, np.zeros(n), lam, eta), np.zeros(n))
    for s in itertools.product((-1, 0, 1), repeat=n):
        s = np.array(s, dtype=np.float64)
        S = np.flatnonzero(s)
        if S.size == 0:
            continue
        AS = A[:, S]
        aS = np.linalg.solve(AS.T @ AS / d + lam * eta * np.eye(S.size), AS.T @ b / d - lam * (1 - eta) * s[S])
        if np.any(np.sign(aS) != s[S]):
            continue
        alpha = np.zeros(n)
        alpha[S] = aS
        val = enet_objective(A, b, alpha, lam, eta)
        if val < best[0]:
            best = (val, alpha)
    return best


def lasso_optimum(A, b, lam):
    """Exact Lasso minimiser by enumerating sign patterns (n <= ~8).

    For a sign pattern s in {-1,0,+1}^n with support S the stationarity condition is
    A_S^T (A_S alpha_S - b) / d + lam s_S = 0; a candidate is kept when its signs agree with s
    and the inactive coordinates satisfy |a_j^T (A alpha - b)| / d <= lam."""
    d, n = A.shape
    best = (lasso_objective(A, b, np.zeros(n), lam), np.zeros(n))
    for s in itertools.product((-1, 0, 1), repeat=n):
        s = np.array(s, dtype=np.float64)
        S = np.flatnonzero(s)
        if S.size == 0:
            continue
        AS = A[:, S]
        G = AS.T @ AS
        if np.linalg.matrix_rank(G) < S.size:
            continue
        aS = np.linalg.solve(G, AS.T @ b - lam * d * s[S])
        if np.any(np.sign(aS) != s[S]):
            continue
        alpha = np.zeros(n)
        alpha[S] = aS
        grad = A.T @ (A @ alpha - b) / d
        if np.any(np.abs(grad) > lam * (1 + 1e-9) + 1e-12):
            continue
        val = lasso_objective(A, b, alpha, lam)
        if val < best[0]:
            best = (val, alpha)
    return best


def svm_dual_optimum(A, y, lam):
    """Exact minimum of the box-constrained SVM dual by enumerating active sets (n <= ~8).

    In t_i = y_i alpha_i in [0,1] the dual is  -(1/n) sum t + t^T Q t / (2 lam n^2) with
    Q = diag(y) A^T A diag(y).  Each coordinate is at 0, at 1, or free; the free block solves
    its stationarity system (least squares when singular); KKT-consistent candidates compete."""
    n = A.shape[1]
    Q = (A * y).T @ (A * y)
    scale = 1.0 / (lam * n * n)

    def val(t):
        return -t.sum() / n + 0.5 * scale * float(t @ Q @ t)

    best = None
    for pat in itertools.product((0, 1, 2), repeat=n):          # 0: lower, 1: upper, 2: free
        pat = np.array(pat)
        t = np.where(pat == 1, 1.0, 0.0)
        F = np.flatnonzero(pat == 2)
        if F.size:
            rhs = np.full(F.size, 1.0 / n) - scale * Q[np.ix_(F, np.flatnonzero(pat != 2))] @ t[pat != 2]
            tF, *_ = np.linalg.lstsq(scale * Q[np.ix_(F, F)], rhs, rcond=None)
            if np.any(tF < -1e-12) or np.any(tF > 1 + 1e-12):
                continue
            t[F] = np.clip(tF, 0.0, 1.0)
        grad = -1.0 / n + scale * (Q @ t)
        ok = (np.all(grad[pat == 0] >= -1e-10) and np.all(grad[pat == 1] <= 1e-10)
              and np.all(np.abs(grad[pat == 2]) <= 1e-9))
        if not ok:
            continue
        cand = val(t)
        if best is None or cand < best[0]:
            best = (cand, y * t)
    assert best is not None
    return best


def best_subset_sum(z, m):
    """max over all subsets of size m of sum z -- the definition of eq. (11) by brute force."""
    return max(sum(z[i] for i in c) for c in itertools.combinations(range(len(z)), m))
