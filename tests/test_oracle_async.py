"""Pins of the oracle's asynchronous schedule (Section II-B, Eq. (c2)-(c4), (d3), (d4)): one active worker per
global step, drawn with the activity probabilities p_i."""
import numpy as np
import pytest
from scipy import stats

from netmax_inputs import workload, iteration_times
from harness import inputs_of, make_oracle
from oracle import policy as opol


def _small(M=6, D=64):
    w = workload("cfg3", M=M, D=D, T=10)
    inp = inputs_of(w)
    return w, inp


def test_activity_by_hand_and_uniform(ora):
    t = np.array([[0, 1, 2.0], [1, 0, 4], [2, 4, 0]])
    P = np.array([[0, .5, .5], [.6, 0, .4], [.3, .7, 0]])
    # Eq. (d3): tbar = (1.5, 2.2, 3.4); Eq. (d4): p_i = (1/tbar_i) / sum (1/tbar)
    f = np.array([1 / 1.5, 1 / 2.2, 1 / 3.4])
    assert np.allclose(ora.activity(t, P), f / f.sum(), rtol=1e-14)
    # the diagonal of t plays no role (d_ii = 0); equal times give every worker the same share
    t2 = np.full((5, 5), 3.0)
    P2 = np.full((5, 5), 0.25) - 0.25 * np.eye(5)
    assert np.allclose(ora.activity(t2, P2), 0.2)
    # a worker that sometimes selects itself: d_ii = 0 in Eq. (d3), so p_ii t_ii adds nothing.
    # tbar = (0.5 * 1 + 0.25 * 2, 2.2, 3.4) = (1.0, 2.2, 3.4) whatever t_00 is
    t3 = t.copy()
    t3[0, 0] = 7.0
    P3 = P.copy()
    P3[0] = [.25, .5, .25]
    f = np.array([1 / 1.0, 1 / 2.2, 1 / 3.4])
    assert np.allclose(ora.activity(t3, P3), f / f.sum(), rtol=1e-14)
    # a missing edge removes that term from the mean iteration time
    adj = np.ones((3, 3), np.uint8) - np.eye(3, dtype=np.uint8)
    adj[0, 2] = 0
    f = np.array([1 / 0.5, 1 / 2.2, 1 / 3.4])
    assert np.allclose(ora.activity(t, P, adj), f / f.sum(), rtol=1e-14)


def test_async_step_is_the_active_workers_row_of_the_synchronous_step(ora):
    """The active worker does what it does in a synchronous iteration with the same counter; nobody else moves."""
    w, inp = _small()
    a, s = make_oracle(w, inp), make_oracle(w, inp)
    a.set_activity(ora.activity(iteration_times(w.links, w.M), inp["P"]))
    seen = set()
    for k in range(40):
        s.X[:], s.V[:] = a.X, a.V
        before_x, before_v = a.X.copy(), a.V.copy()
        i, m = a.async_step(k)
        peers = s.step(k)
        assert peers[i] == m
        assert np.array_equal(a.X[i], s.X[i]) and np.array_equal(a.V[i], s.V[i])
        rest = np.arange(w.M) != i
        assert np.array_equal(a.X[rest], before_x[rest]) and np.array_equal(a.V[rest], before_v[rest])
        seen.add(i)
    assert len(seen) > 1


def test_async_step_is_D_times_the_first_step_update(ora):
    """x^{k+1} = D^k (x^k - alpha g^k), D^k = I + alpha rho gamma_im e_i (e_m - e_i)^T (Eq. (c3), (c4)), plain SGD."""
    w, inp = _small(M=5, D=32)
    a = make_oracle(w, inp, momentum=0.0)
    a.set_activity(np.full(w.M, 1.0 / w.M))
    for k in range(25):
        x = a.X.astype(np.float64)
        i, m = a.async_step(k)
        g = np.zeros_like(x)
        g[i] = a.G[i]
        Dk = np.eye(w.M)
        if m != i:
            gam = 2.0 / (2.0 * a.P[i, m])                     # (d_im + d_mi) / (2 p_im) on the complete graph
            Dk[i, i] -= a.lr * a.rho * gam
            Dk[i, m] += a.lr * a.rho * gam
        assert np.allclose(a.X, Dk @ (x - a.lr * g), rtol=0, atol=2e-6 * np.abs(x).max())


def test_active_worker_and_peer_frequencies(ora):
    w, inp = _small(M=6, D=4)
    a = make_oracle(w, inp)
    p_act = np.array([0.30, 0.05, 0.20, 0.15, 0.10, 0.20])
    a.set_activity(p_act)
    N = 30000
    draws = np.array([ora.async_draw(a.Tact, a.last_act, a.T, a.last, a.seed, k) for k in range(N)])
    cnt = np.bincount(draws[:, 0], minlength=w.M)
    assert stats.chisquare(cnt, p_act * N).pvalue > 1e-3
    i0 = 0                                                     # the most active worker: its peers follow its policy row
    sel = draws[draws[:, 0] == i0, 1]
    pos = a.P[i0] > 0
    assert np.all(np.isin(sel, np.flatnonzero(pos)))
    assert stats.chisquare(np.bincount(sel, minlength=w.M)[pos], a.P[i0][pos] * sel.size).pvalue > 1e-3


def test_one_step_second_moment_matches_Y_P(ora):
    """E ||D^k x||^2 over the draws (i_k, m_k) equals x^T Y_P x (Eq. (d0)-(d2)): ties the two samplers, the weight
    table and the in-place update to the matrix whose second eigenvalue Algorithm 3 minimises."""
    w, inp = _small(M=5, D=16)
    a = make_oracle(w, inp, momentum=0.0, grad_sigma=0.0)
    t = iteration_times(w.links, w.M)
    p_act = ora.activity(t, inp["P"])
    a.set_activity(p_act)
    d = opol.adjacency(w.M)
    Y = opol.y_matrix(np.asarray(a.P), d, a.lr, a.rho, p_act)
    x0 = a.X.copy()
    N = 20000
    acc = np.zeros(w.D)
    sq = np.zeros(w.D)
    for k in range(N):
        a.X[:] = x0
        a.async_step(k)
        n2 = (a.X[:, :w.D].astype(np.float64) ** 2).sum(axis=0)
        acc += n2
        sq += n2 * n2
    mean = acc / N
    sd = np.sqrt(np.maximum(sq / N - mean ** 2, 0.0) / N)
    xs = x0[:, :w.D].astype(np.float64)
    want = np.einsum("ic,ij,jc->c", xs, Y, xs)
    assert np.all(np.abs(mean - want) < 5 * sd + 1e-9 * np.abs(want))
    assert np.all(sd > 0)


def test_async_time_bookkeeping(ora):
    """UpdateTimeVector over a run of global steps: the same as handling the steps one by one with the synchronous
    routine restricted to the active worker, and the geometric closed form for a repeated pair."""
    rng = np.random.default_rng(3)
    M, n, beta = 5, 200, 0.6
    t = rng.uniform(0.5, 4.0, (M, M)).astype(np.float32)
    active = rng.integers(0, M, n).astype(np.int32)
    peers = rng.integers(0, M, n).astype(np.int32)
    ema, clock = np.zeros((M, M), np.float32), np.zeros(M, np.float32)
    ora.update_times_async(active, peers, t, beta, ema, clock)
    ema2, clock2 = np.zeros((M, M), np.float32), np.zeros(M, np.float32)
    for s in range(n):
        # the synchronous routine with every worker but the active one "selecting itself" at zero cost
        peer_all = np.arange(M, dtype=np.int32)
        peer_all[active[s]] = peers[s]
        t_step = t.copy()
        idle = np.arange(M) != active[s]
        t_step[idle, idle] = 0.0
        ora.update_times(peer_all, t_step, beta, ema2, clock2)
    assert np.array_equal(ema, ema2) and np.allclose(clock, clock2, rtol=1e-6)
    # one pair visited k times: (1 - beta^k) t
    k = 9
    ema3 = np.zeros((M, M), np.float32)
    ora.update_times_async(np.full(k, 2, np.int32), np.full(k, 4, np.int32), t, beta, ema3, None)
    assert abs(ema3[2, 4] - (1 - beta ** k) * t[2, 4]) < 1e-5 and np.count_nonzero(ema3) == 1
