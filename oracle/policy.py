"""CPU oracle of NetMax's communication-policy generation (Algorithm 3, "Communication Policy
Generation"; Section III-C; Appendix A for the search intervals; Eq. (d2)-(d4) for Y_P).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Plain numpy / scipy, written to be checked
against the paper by eye: the two grid searches in the paper's order, one linear program per grid
point, the second largest eigenvalue of Y_P, the convergence-time estimate, argmin.

Readings (the listing is garbled in places):
  * the grids are rho = L_rho + k delta_rho (k = 1..K) and tbar = L + r delta (r = 1..R) (the printed
    "rho <- L_rho + delta_rho", "tbar <- L + delta" are loop invariant);
  * L sums over m = 1..M (printed: "i = m");
  * constraint (o3) is taken with >= (a minimum does not exist with >);
  * d_ii = 0: as Eq. (d3) and (o2) are printed, an iteration in which a worker selects itself adds no
    time (the diagonal of the iteration-time matrix is ignored);
  * the linear program min sum_i p_ii s.t. (o2)-(o5) separates by rows and its optimum is not unique.
    Among the optimal points of a row the one with the smallest sum_m (p_im - lb_im)^2 is taken
    (lb_im = alpha rho (d_im + d_mi), the lower bound of (o3)): it is unique, and it is what spreads the
    free probability mass evenly when links are equally fast (uniform policy on a homogeneous network).
    The minimal p_ii comes from scipy's linprog, the least-squares point from its optimality conditions
    by trying every candidate support;
  * epsilon only scales every candidate's T_convergence by the same factor; 1e-3 is used.

Pins (tests/test_oracle_policy_generation.py): the row optimum equals scipy.optimize.linprog's optimal value;
(o2)-(o5) hold; Lemma 1 (Y_P symmetric, rows sum to 1), Lemma 2 (Y_P >= 0), Theorem 3 (largest
eigenvalue 1, second < 1); Y_P of Eq. (d2) equals a Monte-Carlo-free exact expectation of
(D^k)^T D^k over (i, m); a homogeneous network gives the uniform policy.
"""
from __future__ import annotations

import numpy as np
from scipy import optimize


def adjacency(M: int, adj=None) -> np.ndarray:
    if adj is None:
        d = np.ones((M, M), dtype=np.float64) - np.eye(M)
    else:
        d = (np.asarray(adj) != 0).astype(np.float64)
        np.fill_diagonal(d, 0.0)
    return d


def lower_bounds(d: np.ndarray, alpha: float, rho: float) -> np.ndarray:
    """lb_im = alpha rho (d_im + d_mi) for neighbours, 0 elsewhere: constraint (o3)."""
    return alpha * rho * (d + d.T) * d


def tbar_interval(t: np.ndarray, d: np.ndarray, alpha: float, rho: float):
    """[L, U] of Appendix A, Eq. (oa3) and (oa5)."""
    M = t.shape[0]
    L = np.max(alpha * rho / M * np.sum(t * (d + d.T) * d, axis=1))
    U = np.min(np.max(t * d, axis=1) / M)
    return float(L), float(U)


def solve_row(t_row: np.ndarray, d_row: np.ndarray, lb_row: np.ndarray, i: int, target: float):
    """One row of the linear program (lp0): minimise p_ii subject to sum_m t_im p_im = target
    (= M tbar, (o2)), p_im >= lb_im on neighbours (o3), p_im = 0 on non-neighbours (o4), sum_m p_im = 1 (o5);
    among the optimal points the one closest (least squares) to the lower bounds.  Returns p or None."""
    M = t_row.shape[0]
    nb = np.flatnonzero(d_row > 0)
    if nb.size == 0:
        return None
    # variables: p_im for m in nb, then p_ii
    n = nb.size + 1
    cost = np.zeros(n)
    cost[-1] = 1.0
    tt = np.concatenate([t_row[nb], [0.0]])
    A_eq = np.vstack([tt, np.ones(n)])
    b_eq = np.array([target, 1.0])
    bounds = [(lb_row[m], None) for m in nb] + [(0.0, None)]
    res = optimize.linprog(cost, A_eq=A_eq, b_eq=b_eq, bounds=bounds, method="highs")
    if res.status != 0:
        return None
    s_min = max(res.fun, 0.0)
    # second stage: on the optimal face {p_ii = s_min}, the point with the least-squares distance to the lower
    # bounds.  With q = p - lb >= 0 over the neighbours: minimise |q|^2 / 2 subject to sum q = c_mass,
    # sum t q = c_time.  Its optimality (KKT) conditions are q_m = max(0, mu + nu t_m) for two multipliers; the
    # support {q_m > 0} is therefore a set of the fastest or of the slowest links.  Every such support is tried
    # and the one whose multipliers reproduce it is kept.
    lo = np.array([b[0] for b in bounds[:-1]])
    tn = t_row[nb]
    c_mass = 1.0 - s_min - lo.sum()
    c_time = target - float(tn @ lo)
    scale = max(1.0, float(np.abs(tn).max()))
    q = None
    if c_mass <= 1e-13:
        q = np.zeros(nb.size)
    else:
        order = np.argsort(tn, kind="stable")
        best_violation = np.inf
        for j in range(1, nb.size + 1):
            for support in (order[:j], order[nb.size - j:]):
                ts = tn[support]
                G = np.array([[len(ts), ts.sum()], [ts.sum(), (ts * ts).sum()]])
                mult = np.linalg.lstsq(G, np.array([c_mass, c_time]), rcond=None)[0]
                cand = np.zeros(nb.size)
                cand[support] = mult[0] + mult[1] * ts
                off = np.setdiff1d(np.arange(nb.size), support)
                violation = max(abs(cand.sum() - c_mass), abs(float(tn @ cand) - c_time) / scale,
                                float(np.max(-cand, initial=0.0)),
                                float(np.max(mult[0] + mult[1] * tn[off], initial=0.0)))
                if violation < best_violation:
                    best_violation, q = violation, cand
        if best_violation > 1e-9 * max(1.0, c_mass):
            return None
    z = np.concatenate([lo + np.maximum(q, 0.0), [s_min]])
    p = np.zeros(M)
    p[nb] = z[:-1]
    p[i] = max(z[-1], 0.0)
    return p


def solve_lp(t: np.ndarray, d: np.ndarray, alpha: float, rho: float, tbar: float):
    M = t.shape[0]
    lb = lower_bounds(d, alpha, rho)
    P = np.zeros((M, M))
    for i in range(M):
        p = solve_row(t[i], d[i], lb[i], i, M * tbar)
        if p is None:
            return None
        P[i] = p
    return P


def worker_activity(t: np.ndarray, d: np.ndarray, P: np.ndarray) -> np.ndarray:
    """p_i of Eq. (d4) from the mean iteration times of Eq. (d3)."""
    tbar_i = np.sum(t * P * d, axis=1)
    f = 1.0 / tbar_i
    return f / f.sum()


def y_matrix(P: np.ndarray, d: np.ndarray, alpha: float, rho: float, p_act: np.ndarray) -> np.ndarray:
    """Y_P = E[(D^k)^T D^k], Eq. (d2), with gamma_im = (d_im + d_mi) / (2 p_im)."""
    M = P.shape[0]
    gam = np.zeros((M, M))
    sel = (P > 0) & (d > 0)
    gam[sel] = (d + d.T)[sel] / (2.0 * P[sel])
    a1 = p_act[:, None] * P * gam            # p_i p_im gamma_im
    a2 = p_act[:, None] * P * gam ** 2       # p_i p_im gamma_im^2
    np.fill_diagonal(a1, 0.0)
    np.fill_diagonal(a2, 0.0)
    Y = alpha * rho * (a1 + a1.T) - alpha ** 2 * rho ** 2 * (a2 + a2.T)
    diag = 1.0 - 2.0 * alpha * rho * a1.sum(axis=1) + alpha ** 2 * rho ** 2 * (a2.sum(axis=1) + a2.sum(axis=0))
    Y[np.diag_indices(M)] = diag
    return Y


def second_eigenvalue(Y: np.ndarray) -> float:
    w = np.linalg.eigvalsh(0.5 * (Y + Y.T))
    return float(w[-2])


def generate_policy(t, alpha: float, K: int, R: int, adj=None, eps: float = 1e-3):
    """Algorithm 3.  t: M x M iteration times.  Returns dict(P, rho, tbar, lambda2, t_conv) of the best
    candidate, or None if no grid point is feasible."""
    t = np.asarray(t, dtype=np.float64)
    M = t.shape[0]
    d = adjacency(M, adj)
    L_rho, U_rho = 0.0, 0.5 / alpha
    delta_rho = (U_rho - L_rho) / K
    best = None
    for k in range(1, K + 1):
        rho = L_rho + k * delta_rho
        L, U = tbar_interval(t, d, alpha, rho)
        if not L <= U:
            continue
        delta = (U - L) / R
        for r in range(1, R + 1):
            tbar = L + r * delta
            P = solve_lp(t, d, alpha, rho, tbar)
            if P is None:
                continue
            lam2 = second_eigenvalue(y_matrix(P, d, alpha, rho, worker_activity(t, d, P)))
            if not 0.0 < lam2 < 1.0:
                continue
            t_conv = tbar * np.log(eps) / np.log(lam2)
            if best is None or t_conv < best["t_conv"]:
                best = dict(P=P, rho=rho, tbar=tbar, lambda2=lam2, t_conv=float(t_conv))
    return best
