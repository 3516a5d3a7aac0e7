"""Pins of the oracle's momentum-apply + mix step and of the consensus distance."""
import numpy as np
import pytest
import torch


def _setup(rng, M, ld, zero_g=False):
    X = rng.standard_normal((M, ld)).astype(np.float32)
    G = np.zeros((M, ld), np.float32) if zero_g else (0.1 * rng.standard_normal((M, ld))).astype(np.float32)
    V = (0.1 * rng.standard_normal((M, ld))).astype(np.float32)
    return X, G, V


def _policy(rng, M):
    P = rng.random((M, M)) + 0.05
    np.fill_diagonal(P, 0)
    return P / P.sum(1, keepdims=True)


def test_two_step_form_equals_convex_form(ora):
    """Algorithm 2's two updates and the second line of Eq. (c1) are the same map."""
    rng = np.random.default_rng(1)
    M, ld = 6, 192
    X, G, V = _setup(rng, M, ld)
    P = _policy(rng, M)
    w = ora.mix_weights(P, None, 0.1, 0.2)
    peer = np.array([1, 0, 3, 5, 4, 2], np.int32)   # includes a self draw (worker 4)
    Va, Vb = V.copy(), V.copy()
    a = ora.mix(X, G, Va, peer, w, 0.1, 0.9, 1e-4)
    b = ora.mix(X, G, Vb, peer, w, 0.1, 0.9, 1e-4, convex_form=True)
    assert np.array_equal(Va, Vb)
    ulp = np.spacing(np.abs(a))
    assert np.all(np.abs(a - b) <= ulp)
    assert np.array_equal(a[4], (X[4].astype(np.float64) - 0.1 * Va[4].astype(np.float64)).astype(np.float32))


def test_identical_copies_without_gradient_are_a_fixed_point(ora):
    rng = np.random.default_rng(2)
    M, ld = 5, 128
    x = rng.standard_normal(ld).astype(np.float32)
    X = np.tile(x, (M, 1))
    P = _policy(rng, M)
    w = ora.mix_weights(P, None, 0.1, 0.3)
    V = np.zeros_like(X)
    T, last = ora.thresholds(P)
    for it in range(20):
        X = ora.mix(X, np.zeros_like(X), V, ora.sample_peers(T, last, 3, it), w, 0.1, 0.9, 0.0)
        assert np.array_equal(X, np.tile(x, (M, 1)))
        assert ora.consensus_dist(X) == 0.0


def test_two_workers_closed_form_zero_gradient(ora):
    """P = [[0,1],[1,0]], complete graph: w = alpha rho; the mean is kept and x_1 - x_2 shrinks by
    (1 - 2w) per step, so CD_T = (1 - 2w)^(2T) CD_0."""
    rng = np.random.default_rng(3)
    ld, alpha, rho, T = 64, 0.1, 1.5, 10
    X0 = rng.standard_normal((2, ld)).astype(np.float32)
    P = np.array([[0.0, 1.0], [1.0, 0.0]])
    w = ora.mix_weights(P, None, alpha, rho)
    assert w[0, 1] == pytest.approx(alpha * rho)
    X, V = X0.copy(), np.zeros_like(X0)
    Tm, last = ora.thresholds(P)
    cd0 = ora.consensus_dist(X0)
    prev = cd0
    for it in range(T):
        peer = ora.sample_peers(Tm, last, 8, it)
        assert list(peer) == [1, 0]
        X = ora.mix(X, np.zeros_like(X), V, peer, w, alpha, 0.0, 0.0)
        cd = ora.consensus_dist(X)
        assert cd < prev
        prev = cd
    f = 1 - 2 * alpha * rho
    np.testing.assert_allclose(X[0] - X[1], f**T * (X0[0].astype(np.float64) - X0[1]), rtol=0, atol=1e-6)
    np.testing.assert_allclose(X.mean(0), X0.astype(np.float64).mean(0), rtol=0, atol=1e-5)
    assert prev == pytest.approx(f ** (2 * T) * cd0, rel=1e-3)


def test_two_workers_closed_form_scalar_quadratics(ora):
    """f_i(x) = (x - c_i)^2 / 2, mu = 0: s = x_1 + x_2 and d = x_1 - x_2 follow
    s' = [(1-w)(1-a) + w] s + (1-w) a (c_1+c_2),  d' = [(1-w)(1-a) - w] d + (1-w) a (c_1-c_2)."""
    alpha, rho, T = 0.2, 1.0, 40
    w_ = alpha * rho
    c = np.array([1.5, -0.5])
    x = np.array([[0.3], [2.0]], dtype=np.float32)
    X = np.zeros((2, 64), np.float32)
    X[:, :1] = x
    P = np.array([[0.0, 1.0], [1.0, 0.0]])
    w = ora.mix_weights(P, None, alpha, rho)
    V = np.zeros_like(X)
    peer = np.array([1, 0], np.int32)
    s, d = float(x[0, 0]) + float(x[1, 0]), float(x[0, 0]) - float(x[1, 0])
    for _ in range(T):
        G = np.zeros_like(X)
        G[:, 0] = X[:, 0] - c.astype(np.float32)
        X = ora.mix(X, G, V, peer, w, alpha, 0.0, 0.0)
        s = ((1 - w_) * (1 - alpha) + w_) * s + (1 - w_) * alpha * (c[0] + c[1])
        d = ((1 - w_) * (1 - alpha) - w_) * d + (1 - w_) * alpha * (c[0] - c[1])
        assert float(X[0, 0]) + float(X[1, 0]) == pytest.approx(s, abs=2e-5)
        assert float(X[0, 0]) - float(X[1, 0]) == pytest.approx(d, abs=2e-5)
    # geometric closed form of the difference after T steps
    r = (1 - w_) * (1 - alpha) - w_
    d0 = 0.3 - 2.0
    b = (1 - w_) * alpha * (c[0] - c[1])
    assert d == pytest.approx(r**T * d0 + b * (1 - r**T) / (1 - r), abs=1e-5)


def test_expectation_over_the_peer_draw_is_one_step_on_the_consensus_penalty(ora):
    """sum_m q_im x_i'(m) = h_i - alpha rho sum_m (d_im + d_mi)/2 (h_i - x_m): the probabilities
    cancel, which is one SGD step on Eq. (a4)'s penalty term evaluated at (h_i, x_m)."""
    rng = np.random.default_rng(4)
    M, ld, alpha, rho, mu = 5, 64, 0.1, 0.15, 0.9
    X, G, V = _setup(rng, M, ld)
    adj = np.ones((M, M), np.uint8) - np.eye(M, dtype=np.uint8)
    adj[0, 3] = adj[3, 0] = 0
    P = _policy(rng, M) * adj
    P /= P.sum(1, keepdims=True)
    T, last = ora.thresholds(P)
    w = ora.mix_weights(P, adj, alpha, rho)
    Xd, Vd = X.astype(np.float64), V.astype(np.float64)
    Vn = (mu * Vd + G).astype(np.float32).astype(np.float64)
    H = Xd - alpha * Vn
    exp_emp = np.zeros((M, ld))
    for m in range(M):
        peer = np.full(M, m, np.int32)
        out = ora.mix(X, G, V.copy(), peer, w, alpha, mu, 0.0).astype(np.float64)
        exp_emp += P[:, m:m + 1] * out
    want = H.copy()
    for i in range(M):
        for m in range(M):
            if m != i:
                want[i] -= alpha * rho * 0.5 * (int(adj[i, m]) + int(adj[m, i])) * (H[i] - Xd[m])
    np.testing.assert_allclose(exp_emp, want, rtol=0, atol=2e-6)


def test_single_active_worker_matches_the_matrix_form(ora):
    """One worker i with peer m, the others idle (self draw, zero gradient):
    x^{k+1} = D^k (x^k - alpha g^k), D^k = I + alpha rho gamma_im e_i (e_m - e_i)^T (Eq. (c3),(c4))."""
    rng = np.random.default_rng(5)
    M, ld, alpha, rho = 6, 64, 0.05, 0.4
    X, G, _ = _setup(rng, M, ld)
    P = _policy(rng, M)
    w = ora.mix_weights(P, None, alpha, rho)
    i, m = 2, 4
    g = np.zeros_like(G)
    g[i] = G[i]
    peer = np.arange(M, dtype=np.int32)
    peer[i] = m
    out = ora.mix(X, g, np.zeros_like(X), peer, w, alpha, 0.0, 0.0)
    gamma = (1 + 1) / (2 * P[i, m])
    Dk = np.eye(M)
    e_i, e_m = np.eye(M)[i], np.eye(M)[m]
    Dk += alpha * rho * gamma * np.outer(e_i, e_m - e_i)
    want = Dk @ (X.astype(np.float64) - alpha * g.astype(np.float64))
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-6)
    assert np.array_equal(np.delete(out, i, 0), np.delete(X, i, 0))


def test_range_never_grows_without_gradient_and_padding_stays_zero(ora):
    rng = np.random.default_rng(6)
    M, D, ld = 12, 100, 128
    X = np.zeros((M, ld), np.float32)
    X[:, :D] = rng.standard_normal((M, D))
    P = _policy(rng, M)
    w = ora.mix_weights(P, None, 0.1, P[P > 0].min() / 0.4)
    assert w.max() <= 0.25 + 1e-12
    T, last = ora.thresholds(P)
    V = np.zeros_like(X)
    rng_prev = X.max(0) - X.min(0)
    cds = [ora.consensus_dist(X, D)]
    for it in range(60):
        X = ora.mix(X, np.zeros_like(X), V, ora.sample_peers(T, last, 21, it), w, 0.1, 0.9, 0.0)
        r = X.max(0) - X.min(0)
        assert np.all(r <= rng_prev + 1e-7)
        rng_prev = r
        assert np.all(X[:, D:] == 0)
        cds.append(ora.consensus_dist(X, D))
    assert cds[-1] < 0.05 * cds[0]


def test_momentum_apply_reduces_to_torch_sgd_when_rho_is_zero(ora):
    rng = np.random.default_rng(7)
    M, ld, alpha, mu, wd = 3, 64, 0.05, 0.9, 1e-3
    X0 = rng.standard_normal((M, ld)).astype(np.float32)
    P = _policy(rng, M)
    w = ora.mix_weights(P, None, alpha, 0.0)
    assert np.all(w == 0)
    T, last = ora.thresholds(P)
    p = torch.tensor(X0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=alpha, momentum=mu, weight_decay=wd)
    X, V = X0.copy(), np.zeros_like(X0)
    for it in range(10):
        G = (0.1 * rng.standard_normal((M, ld))).astype(np.float32)
        X = ora.mix(X, G, V, ora.sample_peers(T, last, 5, it), w, alpha, mu, wd)
        p.grad = torch.tensor(G, dtype=torch.float64)
        opt.step()
        np.testing.assert_allclose(X, p.detach().numpy(), rtol=0, atol=3e-6)


def test_consensus_distance_equals_pair_sum(ora):
    rng = np.random.default_rng(8)
    M, D, ld = 7, 50, 64
    X = rng.standard_normal((M, ld)).astype(np.float32)
    Xd = X[:, :D].astype(np.float64)
    pair = sum(np.sum((Xd[i] - Xd[m]) ** 2) for i in range(M) for m in range(M)) / (2 * M)
    assert ora.consensus_dist(X, D) == pytest.approx(pair, rel=1e-12)
    assert ora.consensus_dist(np.tile(X[0], (M, 1)), D) == 0.0


def test_fixed_weight_one_half_is_plain_averaging(ora):
    """The gossip / AD-PSGD variant (Section III-D): with weight 1/2 and no gradient two workers that pull from
    each other both land on their mean after one step; the weight does not depend on the policy."""
    rng = np.random.default_rng(11)
    P = np.array([[0.0, 1.0], [1.0, 0.0]])
    w = ora.mix_weights_fixed(P, 0.5)
    assert w[0, 1] == 0.5 and w[1, 0] == 0.5 and w[0, 0] == 0 and w[1, 1] == 0
    X = rng.standard_normal((2, 64)).astype(np.float32)
    out = ora.mix(X, np.zeros_like(X), np.zeros_like(X), np.array([1, 0], np.int32), w, 0.1, 0.0, 0.0)
    mean = X.astype(np.float64).mean(0)
    np.testing.assert_allclose(out[0], mean, atol=1e-7)
    np.testing.assert_allclose(out[1], mean, atol=1e-7)
    assert ora.consensus_dist(out) < 1e-12
    P3 = _policy(rng, 5)
    P3[0, 2] = 0.0
    P3 /= P3.sum(1, keepdims=True)
    w3 = ora.mix_weights_fixed(P3, 0.3)
    assert w3[0, 2] == 0 and np.all(np.diag(w3) == 0) and set(np.unique(w3)) == {0.0, 0.3}


def test_iteration_sequencing_of_the_oracle_class(ora):
    """oracle.Oracle chains the functions pinned above; two closed forms pin the chaining itself.
    (a) Every worker selects itself (p_ii = 1: local step only), plain SGD: after iteration `it` the state is
    x - alpha g(it) with the synthetic gradient OF THAT ITERATION (Algorithm 2: gradient first, then the update).
    (b) Two workers that always select each other, no gradient: the new copies become the current ones, so
    x_1 - x_2 shrinks by (1 - 2 alpha rho) per iteration."""
    rng = np.random.default_rng(12)
    ld, alpha, sigma = 64, 0.1, 0.05
    X0 = rng.standard_normal((3, ld)).astype(np.float32)
    o = ora.Oracle(M=3, ld=ld, D=ld, dims=(), batch=0, lr=alpha, momentum=0.0, weight_decay=0.0, rho=0.2, grad_sigma=sigma,
                   seed=21, P=np.eye(3), X0=X0)
    want = X0.astype(np.float64)
    for it in range(3):
        assert list(o.step(it)) == [0, 1, 2]
        g = ora.synth_grad(3, ld, ld, sigma, 21, it)
        assert np.abs(g).max() > 0
        want = (want - alpha * g.astype(np.float64)).astype(np.float32).astype(np.float64)
        np.testing.assert_allclose(o.X, want, rtol=0, atol=1e-7)
    rho, T = 1.5, 6
    Y0 = rng.standard_normal((2, ld)).astype(np.float32)
    o2 = ora.Oracle(M=2, ld=ld, D=ld, dims=(), batch=0, lr=alpha, momentum=0.0, weight_decay=0.0, rho=rho, grad_sigma=0.0,
                    seed=5, P=np.array([[0.0, 1.0], [1.0, 0.0]]), X0=Y0)
    for it in range(T):
        o2.step(it)
    np.testing.assert_allclose(o2.X[0] - o2.X[1], (1 - 2 * alpha * rho) ** T * (Y0[0].astype(np.float64) - Y0[1]), rtol=0, atol=1e-6)
