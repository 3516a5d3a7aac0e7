"""Host-side policy generation of the library (Algorithm 3) against the oracle.  No GPU needed."""
import numpy as np
import pytest

import paper_2009_05766_amd as nm
from netmax_inputs import iteration_times
from oracle import policy as pol

pytestmark = pytest.mark.filterwarnings("ignore")


def _ring_adj(M, extra=()):
    a = np.zeros((M, M), np.uint8)
    for i in range(M):
        a[i, (i + 1) % M] = a[(i + 1) % M, i] = 1
    for i, m in extra:
        a[i, m] = a[m, i] = 1
    return a


CASES = [
    ("two_tier_10", 8, None, 0.1, 20, 8),
    ("uniform", 8, None, 0.1, 20, 5),
    ("four_group_12", 16, None, 0.05, 40, 6),
    ("three_tier_100_10_1", 32, None, 0.1, 80, 5),
    ("racks8_lognormal", 16, None, 0.1, 40, 6),
    ("lognormal_1p5", 12, None, 0.1, 60, 8),
    ("two_tier_10", 10, "ring", 0.1, 10, 10),
]


@pytest.mark.parametrize("recipe,M,adj,alpha,K,R", CASES)
def test_generated_policy_matches_oracle(recipe, M, adj, alpha, K, R):
    A = _ring_adj(M, [(0, M // 2), (1, M - 2)]) if adj == "ring" else None
    t = iteration_times(recipe, M)
    want = pol.generate_policy(t, alpha, K, R, adj=A)
    if want is None:
        with pytest.raises(nm.NetmaxError) as e:
            nm.netmax_generate_policy(t, alpha, K, R, adj=A)
        assert e.value.code == nm.NETMAX_EINFEASIBLE
        return
    got = nm.netmax_generate_policy(t, alpha, K, R, adj=A)
    assert got["t_conv"] == pytest.approx(want["t_conv"], rel=1e-8)
    assert got["rho"] == pytest.approx(want["rho"], rel=1e-12)
    assert got["tbar"] == pytest.approx(want["tbar"], rel=1e-12)
    assert got["lambda2"] == pytest.approx(want["lambda2"], abs=1e-10)
    np.testing.assert_allclose(got["P"], want["P"], rtol=0, atol=1e-9)
    # and the result can drive the iteration: rows are distributions and the weights satisfy (o3)
    np.testing.assert_allclose(got["P"].sum(1), 1.0, atol=1e-12)
    # strict mode accepts the library's own policy, also with rho rounded to single precision (as netmax_set_policy
    # receives it): links that end on the bound of (o3) have weight 1/2
    thr, last, w = nm.netmax_build_tables(got["P"], A, alpha, float(np.float32(got["rho"])), strict_o3=True)
    assert w.max() <= 0.5 * (1 + 1e-6)


@pytest.mark.parametrize("seed", range(6))
def test_random_time_matrices_match_oracle(seed):
    rng = np.random.default_rng(seed)
    M = int(rng.integers(4, 11))
    t = rng.uniform(0.5, 10.0, (M, M))
    t = np.triu(t, 1) + np.triu(t, 1).T          # symmetric link times
    if seed % 2:
        t[t > 6.0] = 6.0                          # ties among the slow links
    alpha = float(rng.choice([0.05, 0.1, 0.2]))
    K, R = 12 * M, 5
    want = pol.generate_policy(t, alpha, K, R)
    assert want is not None
    got = nm.netmax_generate_policy(t, alpha, K, R)
    assert got["t_conv"] == pytest.approx(want["t_conv"], rel=1e-8)
    np.testing.assert_allclose(got["P"], want["P"], rtol=0, atol=1e-9)
    assert (got["rho"], got["tbar"]) == pytest.approx((want["rho"], want["tbar"]), rel=1e-12)


def test_argument_errors():
    t = iteration_times("two_tier_10", 4)
    with pytest.raises(nm.NetmaxError) as e:
        nm.netmax_generate_policy(t, -0.1, 4, 4)
    assert e.value.code == nm.NETMAX_EINVAL
    bad = t.copy()
    bad[0, 1] = np.nan
    with pytest.raises(nm.NetmaxError):
        nm.netmax_generate_policy(bad, 0.1, 4, 4)
    with pytest.raises(nm.NetmaxError) as e:           # K = 1: rho = 0.5 / alpha leaves no room for (o3)
        nm.netmax_generate_policy(t, 0.1, 1, 4)
    assert e.value.code == nm.NETMAX_EINFEASIBLE


def test_activity_matches_oracle():
    """p_i of Eq. (d3)-(d4): the library's host helper against the oracle, with and without an adjacency mask."""
    import oracle
    rng = np.random.default_rng(5)
    for M in (3, 8, 17):
        t = rng.uniform(0.1, 5.0, (M, M))
        P = rng.uniform(0.0, 1.0, (M, M))
        np.fill_diagonal(P, 0.0)
        adj = (rng.uniform(size=(M, M)) < 0.8).astype(np.uint8)
        adj |= adj.T
        adj[np.arange(M), (np.arange(M) + 1) % M] = 1        # every worker keeps a neighbour
        adj[(np.arange(M) + 1) % M, np.arange(M)] = 1
        np.fill_diagonal(adj, 0)
        P1 = P / P.sum(1, keepdims=True)
        assert np.allclose(nm.netmax_activity(t, P1), oracle.activity(t, P1), rtol=1e-13)
        P2 = P * adj
        P2 = P2 / P2.sum(1, keepdims=True)
        assert np.allclose(nm.netmax_activity(t, P2, adj), oracle.activity(t, P2, adj), rtol=1e-13)
    with pytest.raises(nm.NetmaxError):
        nm.netmax_activity(np.zeros((3, 3)), np.full((3, 3), 1 / 3))


@pytest.mark.parametrize("recipe,M,alpha,K,R", [("two_tier_10", 8, 0.1, 20, 8), ("four_group_12", 16, 0.05, 40, 6),
                                                ("lognormal_1p5", 12, 0.1, 60, 8)])
def test_generated_rows_satisfy_the_optimality_conditions_of_the_second_stage(recipe, M, alpha, K, R):
    """Without enumerating supports (which both the library and the oracle do): on the returned policy every row's
    surplus over the lower bounds of (o3), q_m = p_im - alpha rho (d_im + d_mi), is the least-squares point of the
    optimal face, i.e. q_m = max(0, mu + nu t_im) for two multipliers.  The multipliers are fitted on the links
    with a positive surplus and then have to explain the links without one (mu + nu t_im <= 0 there)."""
    t = iteration_times(recipe, M)
    got = nm.netmax_generate_policy(t, alpha, K, R)
    P, rho = got["P"], got["rho"]
    rows_with_choice = 0
    for i in range(M):
        nb = np.array([m for m in range(M) if m != i])
        q = P[i, nb] - 2.0 * alpha * rho
        assert q.min() > -1e-12
        on = q > 1e-10
        if on.sum() < 2:
            continue
        A = np.stack([np.ones(on.sum()), t[i, nb][on]], axis=1)
        (mu, nu), *_ = np.linalg.lstsq(A, q[on], rcond=None)
        np.testing.assert_allclose(A @ np.array([mu, nu]), q[on], atol=1e-9)
        assert np.all(mu + nu * t[i, nb][~on] <= 1e-9)
        rows_with_choice += 1
    assert rows_with_choice > 0
