"""Pins of the fixed-point thresholds, the peer draw and the mix-weight table."""
import numpy as np
import pytest
from scipy import stats

from netmax_inputs import workload, policy_for, link_speeds, policy_from_speeds, WORKLOAD_NAMES


def _quantised(T, last):
    """q_im implied by stored thresholds: C[m] = T[m] below `last`, 2^32 from `last` on."""
    M = T.shape[0]
    q = np.zeros((M, M), dtype=object)
    for i in range(M):
        C = [int(t) for t in T[i]]
        for m in range(M):
            if m >= last[i]:
                C[m] = 2**32
        prev = 0
        for m in range(M):
            q[i, m] = C[m] - prev
            prev = C[m]
    return q


@pytest.mark.parametrize("name", WORKLOAD_NAMES)
def test_threshold_rows_sum_to_one_and_stay_within_one_lsb(ora, name):
    w = workload(name)
    P, _ = policy_for(w)
    assert np.allclose(P.sum(1), 1.0, atol=1e-12) and np.all(np.diag(P) == 0)
    T, last = ora.thresholds(P)
    q = _quantised(T, last)
    for i in range(w.M):
        assert sum(q[i]) == 2**32                       # exact row sum
        assert all(int(v) >= 0 for v in q[i])           # monotone thresholds
        err = np.array([abs(int(q[i, m]) / 2**32 - P[i, m]) for m in range(w.M)])
        assert err.max() <= 2.0**-32 * (1 + 1e-9) + 1e-15 * w.M   # |q - p| <= 2^-32 (+ double summation)
        assert int(q[i, i]) == 0


def test_zero_probability_entries_are_never_drawn_boundary_sweep(ora):
    P = np.array([[0.0, 0.5, 0.0, 0.5, 0.0],
                  [0.25, 0.0, 0.75, 0.0, 0.0],
                  [0.0, 0.0, 0.0, 0.0, 1.0],
                  [1.0, 0.0, 0.0, 0.0, 0.0],
                  [0.2, 0.2, 0.2, 0.4, 0.0]])
    T, last = ora.thresholds(P)
    assert list(last) == [3, 2, 4, 0, 3]
    for i in range(5):
        us = {0, 1, 2**32 - 1, 2**32 - 2, 2**31}
        for t in T[i]:
            us |= {int(t), max(int(t) - 1, 0), min(int(t) + 1, 2**32 - 1)}
        for u in us:
            m = ora.peer_of_word(T[i], int(last[i]), u)
            assert P[i, m] > 0, (i, u, m)
            # definition: smallest m whose exact cumulative count exceeds u
            C = np.round(np.cumsum(P[i]) * 2**32).astype(object)
            C = [2**32 if k >= last[i] else int(c) for k, c in enumerate(C)]
            assert m == min(k for k in range(5) if u < C[k])


def test_exhaustive_interval_lengths_reproduce_q(ora):
    """Sweeping u over [0, 2^32) the number of words mapped to m is exactly q_im 2^32
    (checked through the interval end points instead of all 2^32 words)."""
    rng = np.random.default_rng(5)
    P = rng.random((6, 6))
    np.fill_diagonal(P, 0)
    P /= P.sum(1, keepdims=True)
    T, last = ora.thresholds(P)
    q = _quantised(T, last)
    for i in range(6):
        lo = 0
        for m in range(6):
            n = int(q[i, m])
            if n == 0:
                continue
            assert ora.peer_of_word(T[i], int(last[i]), lo) == m
            assert ora.peer_of_word(T[i], int(last[i]), lo + n - 1) == m
            lo += n
        assert lo == 2**32


@pytest.mark.parametrize("M", [2, 4, 8])
def test_peer_frequencies_match_policy_chi_square(ora, M):
    rng = np.random.default_rng(M)
    P = rng.random((M, M)) ** 2
    np.fill_diagonal(P, 0)
    P /= P.sum(1, keepdims=True)
    T, last = ora.thresholds(P)
    n_it = 100_000
    counts = np.zeros((M, M), dtype=np.int64)
    for it in range(n_it):
        peer = ora.sample_peers(T, last, 4242, it)
        counts[np.arange(M), peer] += 1
    for i in range(M):
        sel = P[i] > 0
        assert counts[i, ~sel].sum() == 0
        if sel.sum() > 1:
            assert stats.chisquare(counts[i, sel], n_it * P[i, sel]).pvalue > 1e-4
    # draws of different workers are independent: joint table of workers 0 and 1 (M=2 has one cell)


def test_peer_draws_differ_across_workers_and_iterations(ora):
    P = policy_from_speeds(link_speeds("uniform", 16))
    T, last = ora.thresholds(P)
    a = np.array([ora.sample_peers(T, last, 1, it) for it in range(200)])
    assert len({tuple(r) for r in a}) == 200
    assert np.all(a != np.arange(16)[None, :])
    assert np.array_equal(ora.sample_peers(T, last, 1, 17), a[17])
    assert not np.array_equal(ora.sample_peers(T, last, 2, 17), a[17])


@pytest.mark.parametrize("bad", ["neg", "sum", "zero"])
def test_invalid_rows_are_rejected(ora, bad):
    P = np.full((3, 3), 1 / 3)
    if bad == "neg":
        P[1] = [-0.1, 0.6, 0.5]
    elif bad == "sum":
        P[2] = [0.3, 0.3, 0.3]
    else:
        P[0] = 0.0
    with pytest.raises(ValueError):
        ora.thresholds(P)


def test_mix_weight_table(ora):
    """w_im = alpha rho (d_im + d_mi) / (2 p_im) (Algorithm 2, second-step update); constraint
    (o3) p_im > alpha rho (d_im + d_mi) is the same as w_im < 1/2."""
    rng = np.random.default_rng(0)
    M, alpha, rho = 5, 0.1, 0.3
    adj = (rng.random((M, M)) < 0.7).astype(np.uint8)
    adj = np.maximum(adj, adj.T)
    np.fill_diagonal(adj, 0)
    adj[0, 1] = adj[1, 0] = 1
    P = rng.random((M, M)) * adj
    P[P.sum(1) == 0, 0] = 1.0
    P /= P.sum(1, keepdims=True)
    w = ora.mix_weights(P, adj, alpha, rho)
    for i in range(M):
        for m in range(M):
            if i == m or P[i, m] == 0:
                assert w[i, m] == 0
            else:
                theta_coef = (rho / 2) * (int(adj[i, m]) + int(adj[m, i])) / P[i, m]   # Algorithm 2, theta
                assert w[i, m] == pytest.approx(alpha * theta_coef, rel=1e-14)
                assert (P[i, m] > alpha * rho * (int(adj[i, m]) + int(adj[m, i]))) == (w[i, m] < 0.5)
    w_full = ora.mix_weights(P, None, alpha, rho)
    off = (P > 0) & ~np.eye(M, dtype=bool)
    np.testing.assert_allclose(w_full[off], alpha * rho / P[off], rtol=1e-14)
    # a one-way edge: d_01 = 1, d_10 = 0 (the connection matrix need not be symmetric), numbers by hand:
    # w_01 = 0.1 * 0.3 * (1 + 0) / (2 * 0.25) = 0.06, w_02 = 0.1 * 0.3 * 2 / (2 * 0.75) = 0.04,
    # w_10 = 0.1 * 0.3 * (0 + 1) / (2 * 0.5) = 0.03 (p_10 > 0 although d_10 = 0: the weight only reads d)
    adj3 = np.array([[0, 1, 1], [0, 0, 1], [1, 1, 0]], np.uint8)
    P3 = np.array([[0, .25, .75], [.5, 0, .5], [.5, .5, 0]])
    w3 = ora.mix_weights(P3, adj3, alpha, rho)
    assert w3[0, 1] == pytest.approx(0.06, rel=1e-14) and w3[0, 2] == pytest.approx(0.04, rel=1e-14)
    assert w3[1, 0] == pytest.approx(0.03, rel=1e-14)


@pytest.mark.parametrize("name", WORKLOAD_NAMES)
def test_workload_policies_are_feasible(ora, name):
    w = workload(name)
    P, rho = policy_for(w)
    wt = ora.mix_weights(P, None, float(np.float32(w.lr)), rho)
    assert 0 < wt.max() <= 0.25 * (1 + 1e-6)      # rho = p_min / (4 lr)


# ---- iteration-time bookkeeping (Algorithm 2, UpdateTimeVector) -------------------------------------------

def test_update_times_constant_time_closed_form(ora):
    """A link visited n times at a constant time t from a zero start holds (1 - beta^n) t (geometric sum)."""
    M, beta = 4, 0.8
    t = np.full((M, M), 3.0, np.float32)
    ema = np.zeros((M, M), np.float32)
    clock = np.zeros(M, np.float32)
    peer = np.array([1, 2, 3, 0], np.int32)
    for n in range(1, 12):
        ora.update_times(peer, t, beta, ema, clock)
        for i in range(M):
            assert abs(ema[i, peer[i]] - (1 - beta ** n) * 3.0) < 1e-5
    assert np.allclose(clock, 11 * 3.0)
    touched = np.zeros((M, M), bool)
    touched[np.arange(M), peer] = True
    assert np.all(ema[~touched] == 0.0)


def test_update_times_self_selection_and_limits(ora):
    M = 3
    t = np.arange(1, 10, dtype=np.float32).reshape(M, M)
    ema = np.full((M, M), 7.0, np.float32)
    clock = np.zeros(M, np.float32)
    peer = np.array([0, 2, 1], np.int32)             # worker 0 selects itself
    ora.update_times(peer, t, 0.0, ema, clock)    # beta = 0: the latest time replaces the average
    assert ema[0, 0] == 7.0 and ema[1, 2] == t[1, 2] and ema[2, 1] == t[2, 1]
    assert np.array_equal(clock, np.array([t[0, 0], t[1, 2], t[2, 1]], np.float32))
    before = ema.copy()
    ora.update_times(peer, t, 1.0, ema, None)     # beta = 1: the average never moves
    assert np.array_equal(ema, before)
    ema2 = np.zeros((M, M), np.float32)
    ora.update_times(np.array([1, 0, 0], np.int32), t, 0.25, ema2, None)
    assert np.isclose(ema2[0, 1], 0.75 * t[0, 1]) and ema2[1, 0] == np.float32(0.75 * t[1, 0]) and ema2[0, 2] == 0
