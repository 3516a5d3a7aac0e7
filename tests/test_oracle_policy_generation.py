"""Pins of the oracle's policy generation (Algorithm 3)."""
import numpy as np
import pytest
from scipy import optimize

from netmax_inputs import iteration_times
from oracle import policy as pol


def _case(recipe="two_tier_10", M=8, alpha=0.1, rho_frac=0.3, adj=None):
    t = iteration_times(recipe, M)
    d = pol.adjacency(M, adj)
    rho = rho_frac * 0.5 / alpha / (M - 1)      # (o3) needs sum of lower bounds <= 1
    return t, d, alpha, rho


def _ring_adj(M, extra=()):
    a = np.zeros((M, M), np.uint8)
    for i in range(M):
        a[i, (i + 1) % M] = a[(i + 1) % M, i] = 1
    for i, m in extra:
        a[i, m] = a[m, i] = 1
    return a


def test_lower_bounds_are_constraint_o3_and_activity_is_eq_d4():
    """(o3): p_im >= alpha rho (d_im + d_mi) on the edges of worker i, by hand on a graph with a one-way edge;
    Eq. (d3)/(d4): tbar = (1.5, 2.2, 3.4) for the times and policy below, p_i proportional to 1 / tbar_i, so the
    fastest worker is active most often."""
    d = np.array([[0, 1, 1], [0, 0, 1], [1, 1, 0]], float)           # d_01 = 1, d_10 = 0
    lb = pol.lower_bounds(d, 0.1, 0.5)
    want = np.array([[0, 0.05, 0.10], [0, 0, 0.10], [0.10, 0.10, 0]])  # 0.1 * 0.5 * (d_im + d_mi) where d_im = 1
    np.testing.assert_allclose(lb, want, rtol=1e-14)
    t = np.array([[0, 1, 2.0], [1, 0, 4], [2, 4, 0]])
    P = np.array([[0, .5, .5], [.6, 0, .4], [.3, .7, 0]])
    f = np.array([1 / 1.5, 1 / 2.2, 1 / 3.4])
    p_act = pol.worker_activity(t, pol.adjacency(3), P)
    np.testing.assert_allclose(p_act, f / f.sum(), rtol=1e-14)
    assert p_act[0] > p_act[1] > p_act[2]


@pytest.mark.parametrize("recipe,M,adj,rf", [("two_tier_10", 8, None, 0.3), ("lognormal_1p5", 12, None, 0.1),
                                             ("three_tier_100_10_1", 16, None, 0.3), ("two_tier_10", 6, "ring", 0.1)])
def test_row_solution_is_optimal_for_the_linear_program_and_feasible(recipe, M, adj, rf):
    A = _ring_adj(M, [(0, 3)]) if adj == "ring" else None
    t, d, alpha, rho = _case(recipe, M, rho_frac=rf, adj=A)
    L, U = pol.tbar_interval(t, d, alpha, rho)
    assert L < U
    lb = pol.lower_bounds(d, alpha, rho)
    feasible = 0
    for frac in (0.0, 0.1, 0.3, 0.5, 0.9, 1.0):
        tbar = L + frac * (U - L)
        P = pol.solve_lp(t, d, alpha, rho, tbar)
        if P is None:        # L and U are necessary, not sufficient: U ignores the lower bounds of (o3), and the
            continue         # row that fixes L differs from the rows that then lack probability mass
        feasible += 1
        dd = d
        np.testing.assert_allclose(P.sum(1), 1.0, atol=1e-9)                       # (o5)
        np.testing.assert_allclose((t * P * dd).sum(1), M * tbar, rtol=1e-8)      # (o2)
        assert np.all(P[d > 0] >= lb[d > 0] - 1e-10)                               # (o3)
        assert np.all(P[(d == 0) & ~np.eye(M, dtype=bool)] == 0)                   # (o4)
        # the whole program at once (all rows), solved by scipy: same optimal value
        n = M * M
        c = np.zeros(n)
        c[np.arange(M) * M + np.arange(M)] = 1.0
        A_eq = np.zeros((2 * M, n))
        for i in range(M):
            A_eq[i, i * M:(i + 1) * M] = t[i] * dd[i]
            A_eq[M + i, i * M:(i + 1) * M] = 1.0
        b_eq = np.concatenate([np.full(M, M * tbar), np.ones(M)])
        bounds = []
        for i in range(M):
            for m in range(M):
                bounds.append((0.0, None) if i == m else ((lb[i, m], None) if d[i, m] > 0 else (0.0, 0.0)))
        ref = optimize.linprog(c, A_eq=A_eq, b_eq=b_eq, bounds=bounds, method="highs")
        assert ref.status == 0
        assert np.trace(P) == pytest.approx(ref.fun, abs=1e-8)
    assert feasible >= 2


def test_lemmas_hold_for_every_feasible_grid_point():
    """Lemma 1: Y_P symmetric with unit row sums; Lemma 2: Y_P >= 0; Theorem 3: eigenvalues 1 > lambda_2."""
    for recipe, M in (("two_tier_10", 8), ("lognormal_1p5", 10)):
        t, d, alpha, _ = _case(recipe, M)
        for rho in (0.05, 0.2, 0.5):
            L, U = pol.tbar_interval(t, d, alpha, rho)
            if L > U:
                continue
            for frac in (0.2, 0.7, 1.0):
                P = pol.solve_lp(t, d, alpha, rho, L + frac * (U - L))
                if P is None:
                    continue
                pa = pol.worker_activity(t, d, P)
                np.testing.assert_allclose(pa, 1.0 / M, rtol=1e-8)            # equal mean iteration times
                Y = pol.y_matrix(P, d, alpha, rho, pa)
                np.testing.assert_allclose(Y, Y.T, atol=1e-12)
                np.testing.assert_allclose(Y.sum(1), 1.0, atol=1e-10)
                assert Y.min() >= -1e-12
                w = np.linalg.eigvalsh(Y)
                assert w[-1] == pytest.approx(1.0, abs=1e-10) and w[-2] < 1.0 - 1e-9


def test_y_matrix_is_the_exact_expectation_of_DtD():
    """Eq. (d0)-(d2): enumerate the active worker i (probability p_i) and its peer m (probability p_im)."""
    rng = np.random.default_rng(0)
    M, alpha, rho = 6, 0.1, 0.4
    d = pol.adjacency(M, _ring_adj(M, [(0, 2), (1, 4)]))
    P = rng.random((M, M)) * d
    P += np.diag(rng.random(M) * 0.2)                 # some self selection
    P /= P.sum(1, keepdims=True)
    pa = rng.random(M)
    pa /= pa.sum()
    Y = pol.y_matrix(P, d, alpha, rho, pa)
    E = np.zeros((M, M))
    I = np.eye(M)
    for i in range(M):
        for m in range(M):
            if P[i, m] == 0:
                continue
            D = I.copy()
            if m != i:
                gamma = (d[i, m] + d[m, i]) / (2 * P[i, m])
                D += alpha * rho * gamma * np.outer(I[i], I[m] - I[i])      # Eq. (c4)
            E += pa[i] * P[i, m] * D.T @ D
    np.testing.assert_allclose(Y, E, atol=1e-12)


def test_homogeneous_network_gives_a_policy_uniform_over_the_neighbours():
    M, alpha = 8, 0.1
    t = iteration_times("uniform", M, compute=0.05)
    best = pol.generate_policy(t, alpha, K=20, R=5)
    assert best is not None
    P = best["P"]
    off = ~np.eye(M, dtype=bool)
    np.testing.assert_allclose(P[off], P[0, 1], rtol=1e-9)
    np.testing.assert_allclose(np.diag(P), P[0, 0], rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(P.sum(1), 1.0, atol=1e-12)


def test_second_stage_is_the_least_squares_point_of_the_optimal_face():
    """Against a general-purpose constrained minimiser on small rows."""
    rng = np.random.default_rng(3)
    for trial in range(6):
        n = 5
        t_row = np.concatenate([[0.0], rng.uniform(1, 10, n)])
        if trial == 5:
            t_row[1:] = 4.0                                  # equal times: degenerate constraints
        d_row = np.concatenate([[0.0], np.ones(n)])
        lb_row = np.concatenate([[0.0], rng.uniform(0.02, 0.08, n)])
        lo_t, hi_t = float(t_row[1:] @ lb_row[1:]), float(t_row[1:] @ lb_row[1:] + (1 - lb_row.sum()) * t_row[1:].max())
        target = lo_t + rng.uniform(0.2, 0.9) * (hi_t - lo_t)
        p = pol.solve_row(t_row, d_row, lb_row, 0, target)
        assert p is not None
        s_min = p[0]
        rows = [np.ones(n)] if trial == 5 else [np.ones(n), t_row[1:]]
        rhs = [1 - s_min] if trial == 5 else [1 - s_min, target]
        ref = optimize.minimize(lambda z: 0.5 * np.sum((z - lb_row[1:]) ** 2), p[1:] * 0 + (1 - s_min) / n,
                                jac=lambda z: z - lb_row[1:], method="trust-constr",
                                constraints=[optimize.LinearConstraint(np.vstack(rows), rhs, rhs)],
                                bounds=optimize.Bounds(lb_row[1:], np.inf), options={"gtol": 1e-12, "xtol": 1e-14})
        np.testing.assert_allclose(p[1:], ref.x, atol=2e-6)
        assert 0.5 * np.sum((p[1:] - lb_row[1:]) ** 2) <= ref.fun + 1e-9


def test_generated_policy_prefers_fast_links_and_is_feasible_for_the_iteration():
    M, alpha = 8, 0.1
    t = iteration_times("two_tier_10", M)
    best = pol.generate_policy(t, alpha, K=20, R=8)
    assert best is not None and 0 < best["lambda2"] < 1 and 0 < best["rho"] <= 0.5 / alpha
    P = best["P"]
    intra = P[0, 1:4].mean()
    inter = P[0, 4:].mean()
    assert intra > inter                                   # fast links are chosen more often
    # every selectable pair satisfies (o3), i.e. mix weight <= 1/2
    off = (P > 0) & ~np.eye(M, dtype=bool)
    assert np.all(alpha * best["rho"] * 2 / (2 * P[off]) <= 0.5 + 1e-9)
    # exhaustive check of the argmin over the grid
    d = pol.adjacency(M)
    cands = []
    for k in range(1, 21):
        rho = k * (0.5 / alpha) / 20
        L, U = pol.tbar_interval(t, d, alpha, rho)
        if L > U:
            continue
        for r in range(1, 9):
            tbar = L + r * (U - L) / 8
            Pc = pol.solve_lp(t, d, alpha, rho, tbar)
            if Pc is None:
                continue
            lam = pol.second_eigenvalue(pol.y_matrix(Pc, d, alpha, rho, pol.worker_activity(t, d, Pc)))
            if 0 < lam < 1:
                cands.append(tbar * np.log(1e-3) / np.log(lam))
    assert best["t_conv"] == pytest.approx(min(cands), rel=1e-9)


def test_search_intervals():
    """Appendix A: U_rho = 0.5 / alpha; L from (o2)+(o3); U from the slowest neighbour."""
    M, alpha, rho = 5, 0.2, 0.3
    t = iteration_times("two_tier_10", M)
    d = pol.adjacency(M)
    L, U = pol.tbar_interval(t, d, alpha, rho)
    Li = [alpha * rho / M * sum(t[i, m] * 2 for m in range(M) if m != i) for i in range(M)]
    Ui = [max(t[i, m] for m in range(M) if m != i) / M for i in range(M)]
    assert L == pytest.approx(max(Li)) and U == pytest.approx(min(Ui))
