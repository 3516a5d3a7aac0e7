"""Pins of the oracle's local gradient: finite differences and torch.autograd in fp64."""
import numpy as np
import pytest
import torch

from netmax_inputs import f32_to_bf16_bits, bf16_bits_to_f32


def _problem(rng, dims, n, B, bf16=False):
    D = sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1))
    params = (rng.standard_normal(D) * 0.3).astype(np.float32)
    feats = rng.standard_normal((n, dims[0])).astype(np.float32)
    if bf16:
        feats = f32_to_bf16_bits(feats)
    labels = rng.integers(0, dims[-1], n).astype(np.int32)
    idx = rng.integers(0, n, B).astype(np.int32)
    return params, feats, labels, idx


def _torch_loss_grad(dims, params, feats_f32, labels, idx):
    p = torch.tensor(params, dtype=torch.float64, requires_grad=True)
    a = torch.tensor(feats_f32[idx], dtype=torch.float64)
    o = 0
    for l in range(len(dims) - 1):
        W = p[o:o + dims[l] * dims[l + 1]].reshape(dims[l], dims[l + 1])
        o += dims[l] * dims[l + 1]
        b = p[o:o + dims[l + 1]]
        o += dims[l + 1]
        a = a @ W + b
        if l + 2 < len(dims):
            a = torch.relu(a)
    loss = torch.nn.functional.cross_entropy(a, torch.tensor(labels[idx], dtype=torch.long))
    loss.backward()
    return float(loss.detach()), p.grad.numpy()


@pytest.mark.parametrize("dims", [(8, 3), (6, 5, 4), (7, 6, 5, 3), (256, 10)])
def test_gradient_matches_torch_autograd_fp64(ora, dims):
    rng = np.random.default_rng(len(dims) * 100 + dims[0])
    params, feats, labels, idx = _problem(rng, dims, 40, 12)
    g, loss = ora.grad_mlp(dims, params, feats, labels, idx)
    tl, tg = _torch_loss_grad(dims, params, feats, labels, idx)
    assert loss == pytest.approx(tl, rel=1e-12)
    np.testing.assert_allclose(g, tg, rtol=1e-6, atol=1e-9)


def test_gradient_with_bf16_features_matches_torch(ora):
    rng = np.random.default_rng(9)
    dims = (16, 8, 4)
    params, feats, labels, idx = _problem(rng, dims, 30, 10, bf16=True)
    g, loss = ora.grad_mlp(dims, params, feats, labels, idx)
    tl, tg = _torch_loss_grad(dims, params, bf16_bits_to_f32(feats), labels, idx)
    assert loss == pytest.approx(tl, rel=1e-12)
    np.testing.assert_allclose(g, tg, rtol=1e-6, atol=1e-9)


@pytest.mark.parametrize("dims", [(5, 3), (4, 6, 3)])
def test_gradient_matches_central_finite_differences(ora, dims):
    rng = np.random.default_rng(17 + len(dims))
    params, feats, labels, idx = _problem(rng, dims, 20, 6)
    # keep pre-activations away from the ReLU kink: quantise parameters to multiples of 2^-6 so that
    # +-2^-9 perturbations are exact in float
    params = (np.round(params * 64) / 64).astype(np.float32)
    g, _ = ora.grad_mlp(dims, params, feats, labels, idx)
    h = 2.0 ** -9
    for j in range(params.size):
        pp, pm = params.copy(), params.copy()
        pp[j] += np.float32(h)
        pm[j] -= np.float32(h)
        lp = ora.grad_mlp(dims, pp, feats, labels, idx)[1]
        lm = ora.grad_mlp(dims, pm, feats, labels, idx)[1]
        fd = (lp - lm) / (2 * h)
        assert g[j] == pytest.approx(fd, rel=2e-3, abs=2e-5), j


def test_softmax_regression_closed_form(ora):
    """One layer: grad W = X^T (softmax(XW+b) - onehot) / B, grad b = column sums / B."""
    rng = np.random.default_rng(23)
    dims = (12, 5)
    params, feats, labels, idx = _problem(rng, dims, 25, 9)
    g, loss = ora.grad_mlp(dims, params, feats, labels, idx)
    W = params[:60].reshape(12, 5).astype(np.float64)
    b = params[60:65].astype(np.float64)
    Xb = feats[idx].astype(np.float64)
    z = Xb @ W + b
    p = np.exp(z - z.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    y = labels[idx]
    assert loss == pytest.approx(-np.log(p[np.arange(9), y]).mean(), rel=1e-12)
    p[np.arange(9), y] -= 1
    np.testing.assert_allclose(g[:60].reshape(12, 5), Xb.T @ p / 9, rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(g[60:], p.sum(0) / 9, rtol=1e-6, atol=1e-9)


def test_all_workers_wrapper_uses_each_workers_shard_and_zeroes_padding(ora):
    rng = np.random.default_rng(31)
    dims, M, B = (6, 4, 3), 3, 5
    D = 6 * 4 + 4 + 4 * 3 + 3
    ld = 64
    shard_off = np.array([0, 7, 19, 30], dtype=np.int64)
    feats = rng.standard_normal((30, 6)).astype(np.float32)
    labels = rng.integers(0, 3, 30).astype(np.int32)
    X = np.zeros((M, ld), np.float32)
    X[:, :D] = rng.standard_normal((M, D)) * 0.3
    idx = ora.sample_batch(M, B, shard_off, 3, 0)
    G, loss = ora.local_grad(dims, X, feats, labels, shard_off, idx)
    for i in range(M):
        s, e = shard_off[i], shard_off[i + 1]
        g, l = ora.grad_mlp(dims, X[i], feats[s:e], labels[s:e], idx[i])
        assert np.array_equal(G[i, :D], g) and loss[i] == l
        assert np.all(G[i, D:] == 0)


def test_bf16_rounding_matches_torch_cast(ora):
    rng = np.random.default_rng(3)
    xs = np.concatenate([rng.standard_normal(2000) * 10.0 ** rng.integers(-6, 6, 2000),
                         [1.0 + 2**-8, 1.0 + 3 * 2**-8, -(1.0 + 2**-8), 0.0, 2.0**-130, 1.0 + 2**-8 + 2**-20]])
    for x in xs:
        want = float(torch.tensor(np.float32(x)).to(torch.bfloat16).to(torch.float64))
        assert ora.round_bf16(float(x)) == want


class _Bf16Matmul(torch.autograd.Function):
    """A @ W with both operands cast to bfloat16 by torch, in the forward product and in both
    backward products; the chain rule around it is left to autograd."""

    @staticmethod
    def forward(ctx, a, w):
        r = lambda t: t.to(torch.float32).to(torch.bfloat16).to(torch.float64)
        ctx.save_for_backward(r(a), r(w))
        return r(a) @ r(w)

    @staticmethod
    def backward(ctx, gz):
        r = lambda t: t.to(torch.float32).to(torch.bfloat16).to(torch.float64)
        a, w = ctx.saved_tensors
        return r(gz) @ w.T, a.T @ r(gz)


@pytest.mark.parametrize("dims", [(16, 4), (24, 12, 5), (20, 16, 12, 6)])
def test_bf16_operand_mode_matches_torch_autograd_with_bf16_cast_products(ora, dims):
    rng = np.random.default_rng(sum(dims))
    params, feats, labels, idx = _problem(rng, dims, 40, 13, bf16=True)
    g, loss = ora.grad_mlp(dims, params, feats, labels, idx, operands_bf16=True)
    p = torch.tensor(params, dtype=torch.float64, requires_grad=True)
    a = torch.tensor(bf16_bits_to_f32(feats)[idx], dtype=torch.float64)
    o = 0
    for l in range(len(dims) - 1):
        W = p[o:o + dims[l] * dims[l + 1]].reshape(dims[l], dims[l + 1])
        o += dims[l] * dims[l + 1]
        b = p[o:o + dims[l + 1]]
        o += dims[l + 1]
        a = _Bf16Matmul.apply(a, W) + b
        if l + 2 < len(dims):
            a = torch.relu(a)
    tl = torch.nn.functional.cross_entropy(a, torch.tensor(labels[idx], dtype=torch.long))
    tl.backward()
    assert loss == pytest.approx(float(tl.detach()), rel=1e-12)
    np.testing.assert_allclose(g, p.grad.numpy(), rtol=1e-6, atol=1e-9)
    # and it differs measurably from the exact-arithmetic gradient
    g_exact, _ = ora.grad_mlp(dims, params, feats, labels, idx)
    assert 1e-4 < np.linalg.norm(g - g_exact) / np.linalg.norm(g_exact) < 0.1


@pytest.mark.parametrize("dims,bf16", [((6, 5, 4), False), ((7, 6, 5, 3), False), ((20, 16, 12, 6), True)])
def test_hidden_pre_activations_match_torch(ora, dims, bf16):
    """ora_hidden_mlp against a forward pass written with torch (fp64 matmuls; in the bf16 mode both operands of
    every product cast by torch): layer order, bias included, value before the ReLU."""
    rng = np.random.default_rng(5 + sum(dims))
    params, feats, labels, idx = _problem(rng, dims, 40, 11, bf16=bf16)
    zs = ora.hidden_mlp(dims, params, feats, idx, operands_bf16=bf16)
    assert len(zs) == len(dims) - 2
    r = (lambda t: t.to(torch.float32).to(torch.bfloat16).to(torch.float64)) if bf16 else (lambda t: t)
    p = torch.tensor(params, dtype=torch.float64)
    a = torch.tensor((bf16_bits_to_f32(feats) if bf16 else feats)[idx], dtype=torch.float64)
    o = 0
    for l in range(len(dims) - 2):
        W = p[o:o + dims[l] * dims[l + 1]].reshape(dims[l], dims[l + 1])
        o += dims[l] * dims[l + 1]
        b = p[o:o + dims[l + 1]]
        o += dims[l + 1]
        z = r(a) @ r(W) + b
        assert zs[l].shape == (11, dims[l + 1])
        np.testing.assert_allclose(zs[l], z.numpy(), rtol=1e-12, atol=1e-13)
        assert (zs[l] < 0).any() and (zs[l] > 0).any()
        a = torch.relu(z)


def test_all_workers_hidden_wrapper(ora):
    rng = np.random.default_rng(41)
    dims, M, B = (6, 5, 4, 3), 3, 5
    D = sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(3))
    shard_off = np.array([0, 7, 19, 30], dtype=np.int64)
    feats = rng.standard_normal((30, 6)).astype(np.float32)
    X = np.zeros((M, 128), np.float32)
    X[:, :D] = rng.standard_normal((M, D)) * 0.3
    idx = ora.sample_batch(M, B, shard_off, 3, 0)
    Z = ora.local_hidden(dims, X, feats, shard_off, idx)
    for i in range(M):
        zs = ora.hidden_mlp(dims, X[i], feats[shard_off[i]:shard_off[i + 1]], idx[i])
        for l in range(2):
            assert np.array_equal(Z[l][i], zs[l])
